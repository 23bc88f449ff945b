#!/usr/bin/env python3
"""Benchmark of the linked-operator-chain CNN path on one MI355X.

One "step" = one forward pass of the whole planned chain sequence over one batch of synthetic input
that is already resident in HBM.  Prints ONE JSON line.  The headline workload is config 3
(VGG-16-style, batch 32, bf16 MFMA / fp32 accumulate, linked + split): the largest single-GPU
configuration and the compute-bound regime in which the MFMA roofline is meaningful.

Fixed policy, no minimum over variants: the headline is the path at link level 3, the deepest linking the library has, partitions profiled per chain
(xenos_plan_tune), one launch per chain, with TWO passes in flight: step k is enqueued on stream k % 2 with
the workspace and output of that stream (xenos_run on the bound workspace, xenos_run_with on the second
one), so consecutive steps, which work on independent batches, overlap: the kernels of one fill the
compute units that the last round of tiles of the other leaves idle, and the gap behind a dependent launch
is covered.  `value` is images/s of K such steps between two device synchronisations.  The same K steps
one after the other on one stream (the latency of a pass), HIP-graph replay of the same plan
(xenos_run_graph) and the other link levels (2, U1, U0) are reported beside it.  The roofline of the
dominant kernel is measured on launches that have the chip to themselves (one pass at a time, HIP events
around every launch); its HBM traffic is counted by rocprofv3 child processes started before this process touches
the GPU (measure_traffic).  The other workloads report images/s of one pass at a time at every link level, and of two
passes in flight beside it.  Batch-1 workloads are timed over at least 1000 passes whatever --steps says.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (config, batch, compute)
    "vgg16_n32_bf16": (3, 32, 1),
    "resnet18_n32_bf16": (2, 32, 1),
    "resnet18_n1_bf16": (2, 1, 1),
    "mobilenet_n1_bf16": (1, 1, 1),
    "mobilenet_n1_f32": (1, 1, 0),
    "squeezenet_n1_bf16": (4, 1, 1),
    "squeezenet_n1_f32": (4, 1, 0),
    "squeezenet_n32_bf16": (4, 32, 1),
    "squeezenet_n32_f32": (4, 32, 0),
    "single_chain_n1_f32": (0, 1, 0),
    "shufflenet_n1_bf16": (5, 1, 1),
    "shufflenet_n32_bf16": (5, 32, 1),
}
PEAK = {1: 2500.0, 0: 157.3}          # dense MFMA TFLOP/s: bf16, fp32
HBM_PEAK = 8000.0                     # GB/s
LINK_NAMES = {3: "linked_deep", 2: "linked", 1: "U1", 0: "U0"}   # linked_deep: + the chains whose intermediate stays on chip
HEADLINE_LINK = 3
IN_FLIGHT = 2                         # passes of the headline policy that are in flight at a time (one stream each)
MIN_PASSES_BATCH1 = 1000


def time_steps(sess, torch, steps, warmup, graph=False):
    """K forward passes.  graph=False enqueues the kernels one by one (xenos_run); graph=True replays the HIP graph
    of the same chain sequence (xenos_run_graph)."""
    run = sess.run_graph if graph else sess.run
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


_STREAMS = []


def pick_streams(X, torch, n=IN_FLIGHT, tries=8):
    """The streams the steps in flight run on, created once per process.  HIP serves a process's streams from a few
    hardware queues (four by default) and two streams that share a queue run their kernels one after the other, so each
    new stream is checked against the ones already chosen with a probe that has nothing to do with the workload: a small
    MFMA-only kernel on eight compute units, once on each of the two streams at a time; a stream on whose queue the pair
    takes as long as two such kernels in a row is dropped and the next one is tried.  Returns a note for the JSON line."""
    if len(_STREAMS) >= n:
        return "kept"
    hw = dict(X.MI355X)
    hw["num_cu"] = 8
    nout = 8192 * hw["num_cu"]
    outs = [torch.empty(nout, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cur = torch.cuda.current_stream()

    def pair_ms(sa, sb):
        # one probe kernel on each stream (both behind e0), or two in a row on sa when sb is None
        torch.cuda.synchronize()
        e0.record()
        for j, st in enumerate((sa, sb if sb is not None else sa)):
            st.wait_event(e0)
            X.xenos_probe_mfma(outs[j].data_ptr(), nout, 4000, st.cuda_stream, hw=hw)
            cur.wait_stream(st)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    _STREAMS.append(torch.cuda.Stream())
    pair_ms(_STREAMS[0], None)                                          # warm-up
    serial = pair_ms(_STREAMS[0], None)
    dropped = 0
    while len(_STREAMS) < n and dropped < tries:
        cand = torch.cuda.Stream()
        if all(min(pair_ms(st, cand), pair_ms(st, cand)) < 0.75 * serial for st in _STREAMS):
            _STREAMS.append(cand)
        else:
            dropped += 1
    while len(_STREAMS) < n:                                           # (no independent queue found: the steps then simply run in turn)
        _STREAMS.append(torch.cuda.Stream())
    return "%d streams on separate hardware queues (probe pairs overlap), %d candidate streams dropped" % (n, dropped)


def time_in_flight(sess, lanes, torch, steps, warmup):
    """K forward passes with 1 + len(lanes) of them in flight: pass k goes to stream j = k % (1 + len(lanes)) with the
    input, workspace and output of that stream (the session's own for j = 0, a lane's otherwise), so a pass follows
    the pass before it on its stream and overlaps the passes of the other streams.  Returns (ms per pass between an event
    every stream waits for and one that waits for every stream, wall-clock ms per pass between two synchronisations)."""
    runs = [sess.run] + [l.run for l in lanes]
    while len(_STREAMS) < len(runs):      # created once per process, one after the other, and reused by every measurement
        _STREAMS.append(torch.cuda.Stream())
    streams = _STREAMS[:len(runs)]

    def go(n):
        for k in range(n):
            j = k % len(runs)
            with torch.cuda.stream(streams[j]):
                runs[j]()

    go(warmup)
    torch.cuda.synchronize()
    cur = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for st in streams:
        st.wait_event(e0)
    go(steps)
    for st in streams:
        cur.wait_stream(st)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


def time_each_step(sess, torch, steps):
    """Durations of single passes (ms): an event between consecutive passes, for the median and the spread."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record()
    for i in range(steps):
        sess.run()
        evs[i + 1].record()
    torch.cuda.synchronize()
    return np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])


def time_chains(sess, torch, steps):
    """Per-chain times between HIP events recorded around every launch on the launch stream (ms, average over `steps`
    instrumented passes), and the span of such a pass from its first event to its last."""
    n = sess.info["n_chains"]
    tot = np.zeros(n)
    span = 0.0
    for _ in range(steps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        evs[0].record()
        for i in range(n):
            sess.run_chain(i)
            evs[i + 1].record()
        torch.cuda.synchronize()
        tot += np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(n)])
        span += evs[0].elapsed_time(evs[n])
    return tot / steps, span / steps


TUNE = True     # profiling-driven partition choice (xenos_plan_tune) before timing; --no-tune keeps the cost model's choice


def chain_label(c):
    if c["kind"] != "conv":
        return c["kind"]
    if c.get("halo"):
        return "conv3x3_kernel"
    return {"stem": "stem kernel", "pair": "conv_pair_kernel", "stream": "fc_stream_kernel", "pwdw": "pwdw_kernel", "fire": "fire_kernel",
            "vector": "dwpw_kernel" if c.get("dw_linked") else "conv_kernel", "scalar": "conv_kernel"}.get(c.get("loader"), "conv_kernel")


def run_workload(name, steps, warmup, links=(3,), chains=False, wg=None, X=None, torch=None, graph=None):
    cfg, batch, compute = WORKLOADS[name]
    g = graph if graph is not None else wg.build(cfg, batch)
    passes = steps if batch > 1 else max(steps, MIN_PASSES_BATCH1)
    out = {"workload": name, "config": cfg, "batch": batch, "dtype": "bf16" if compute else "f32",
           "gflop": wg.conv_fc_flops(g) / 1e9, "passes_timed": passes}
    for link in links:
        s = X.Session(g, link=link, split=1, compute=compute)
        s.set_input(g.x)
        retuned = s.tune(reps=5) if TUNE else 0
        ms, wall = time_steps(s, torch, passes, warmup, graph=False)
        ms_graph, _ = time_steps(s, torch, passes, warmup, graph=True)
        each = time_each_step(s, torch, passes)
        lanes = [s.lane() for _ in range(IN_FLIGHT - 1)]
        for l in lanes:
            l.x.copy_(s.x)
        ms_fl, wall_fl = time_in_flight(s, lanes, torch, passes, warmup)
        del lanes
        rec = {"ms_per_step_in_flight": ms_fl, "wall_ms_per_step_in_flight": wall_fl, "passes_in_flight": IN_FLIGHT,
               "images_per_s_in_flight": batch / ms_fl * 1e3,
               "ms_per_step": ms, "wall_ms_per_step": wall, "ms_per_step_graph_replay": ms_graph, "launch": "xenos_run (one launch per chain)",
               "ms_per_step_median": float(np.median(each)), "ms_per_step_min": float(each.min()), "ms_per_step_p90": float(np.percentile(each, 90)),
               "images_per_s": batch / ms * 1e3, "images_per_s_graph_replay": batch / ms_graph * 1e3,
               "tuned": bool(TUNE), "chains_retuned": retuned,
               "tflops": out["gflop"] / ms, "n_chains": s.info["n_chains"],
               "algorithmic_hbm_mb": s.info["hbm_bytes"] / 1e6,
               "algorithmic_gb_per_s": s.info["hbm_bytes"] / ms / 1e6}
        if chains:
            # An event between two launches keeps the second from being dispatched behind the first: the instrumented pass
            # is longer than the plain one by a gap per launch.  That gap is measured here, (instrumented pass - plain
            # pass) / launches, and taken off every chain's time between its events, so that the chain times add up to the
            # plain pass (rocprofv3's kernel durations of the same plan agree with them; see profiles/).
            raw, span = time_chains(s, torch, max(3, min(steps, 20) // 2))
            gap = max(0.0, (span - ms) / len(raw))
            cms = np.maximum(raw - gap, 0.6 * raw)          # (a launch of a few microseconds keeps at least 60 % of what its events read)
            rec["event_gap_ms_per_launch"] = gap
            rec["instrumented_pass_ms"] = span
            rec["chains"] = [dict(i=c["i"], name=c["name"], kind=c["kind"], kernel=chain_label(c), ms=float(cms[c["i"]]),
                                  ms_between_events=float(raw[c["i"]]), gflop=c["flops"] / 1e9,
                                  mb=(c["bytes_in"] + c["bytes_w"] + c["bytes_out"] + c["bytes_res"]) / 1e6,
                                  mode=c.get("mode"), tile=[c.get("bm"), c.get("bn")] if c["kind"] == "conv" else None,
                                  loader=c.get("loader"), halo=c.get("halo", 0), ksplit=c.get("ksplit", 1))
                             for c in s.info["chains"]]
        out[LINK_NAMES[link]] = rec
        s.close()
        del s
        torch.cuda.empty_cache()
    return out, g


def layer_table(chains, compute):
    """Per-chain roofline rows: the bound is the roof the chain's arithmetic intensity puts it under."""
    ridge = PEAK[compute] * 1e3 / HBM_PEAK          # flop per byte
    rows = []
    for c in chains:
        ai = c["gflop"] * 1e3 / max(c["mb"], 1e-9)
        bound = "mfma" if (c["kind"] == "conv" and ai >= ridge) else "hbm"
        tf, gbs = c["gflop"] / c["ms"], c["mb"] / c["ms"]
        rows.append({"chain": c["name"], "kernel": c["kernel"], "us": round(c["ms"] * 1e3, 2), "gflop": round(c["gflop"], 3), "mb": round(c["mb"], 3),
                     "tflops": round(tf, 1), "gb_per_s": round(gbs, 1), "bound": bound,
                     "frac": round(tf / PEAK[compute] if bound == "mfma" else gbs / HBM_PEAK, 4)})
    return rows


def attainable(X, torch):
    """What this GPU attains on the two roofs, measured here with the library's probe kernels: an MFMA-only loop (bf16
    32x32x16, no memory instruction in the loop) and a streaming read of 1 GiB of device memory."""
    nout = 8192 * X.MI355X["num_cu"]
    out = torch.empty(nout, dtype=torch.uint8, device="cuda:0")
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
    st = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    res = {}
    # the sustained MFMA rate depends on the operand values (the clock follows the switching activity): the loop is timed on
    # small structured operands, on pseudo-random dense ones, and on pseudo-random ones with half of the pixel operand zero,
    # which is what a convolution behind a ReLU multiplies
    for data, key in ((0, "mfma_loop_tflops_bf16"), (1, "mfma_loop_tflops_bf16_random_operands"), (2, "mfma_loop_tflops_bf16_relu_like_operands")):
        flops = X.xenos_probe_mfma(out.data_ptr(), nout, 2000, st, data=data)              # warm-up
        torch.cuda.synchronize()
        e0.record()
        flops = X.xenos_probe_mfma(out.data_ptr(), nout, 20000, st, data=data)
        e1.record()
        torch.cuda.synchronize()
        res[key] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    nbytes = src.numel() * 4
    X.xenos_probe_read(src.data_ptr(), nbytes, out.data_ptr(), nout, st)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        X.xenos_probe_read(src.data_ptr(), nbytes, out.data_ptr(), nout, st)
    e1.record()
    torch.cuda.synchronize()
    res["stream_read_gb_per_s"] = 5 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, out
    torch.cuda.empty_cache()
    return res


def measure_traffic(workload, link):
    """HBM bytes per launch of the dominant kernel, measured for this run: four child processes under rocprofv3 (one
    counter each: FETCH_SIZE and WRITE_SIZE, in KiB per dispatch, for a plain 256 MiB device copy and for four passes of the
    workload planned and tuned as the timed one is), the workload's counters scaled by what the same counters read for the
    copy.  Called before this process touches the GPU.  Returns (bytes per launch or None, a note saying what was done)."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    if shutil.which("rocprofv3") is None:
        return None, "rocprofv3 not found"
    tmp = tempfile.mkdtemp(prefix="xenos_traffic_", dir="/tmp")
    env = dict(os.environ, TMPDIR="/tmp")

    def run(tag, counter, prog_args):
        d = os.path.join(tmp, tag)
        cmd = ["rocprofv3", "--pmc", counter, "--output-format", "csv", "-d", d, "--", sys.executable, os.path.join(ROOT, "bench.py")] + prog_args
        # (a child that does not finish is ended with its whole process group: the profiler starts the program as its child)
        pr = subprocess.Popen(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, start_new_session=True)
        try:
            out, err = pr.communicate(timeout=90)
        except subprocess.TimeoutExpired:
            import signal
            os.killpg(pr.pid, signal.SIGKILL)
            pr.communicate()
            raise RuntimeError("%s: no result within 90 s" % tag)
        r = argparse.Namespace(returncode=pr.returncode, stdout=out, stderr=err)
        if r.returncode != 0:
            raise RuntimeError("%s: rc %d: %s" % (tag, r.returncode, (r.stderr or r.stdout)[-300:]))
        files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
        if not files:
            raise RuntimeError("%s: no counter file" % tag)
        by = {}
        for row in csv.DictReader(open(max(files, key=os.path.getmtime))):
            if row["Counter_Name"] != counter:
                continue
            e = by.setdefault(int(row["Dispatch_Id"]), [row["Kernel_Name"], 0.0])
            e[1] += float(row["Counter_Value"])
        info = None
        for ln in r.stdout.splitlines():
            if ln.startswith("{"):
                info = json.loads(ln)
        return [by[k] for k in sorted(by)], info

    try:
        scale = {}
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            rows, info = run("cal_" + counter, counter, ["--calibrate-copy"])
            cp = [v for k, v in rows if "copy" in k.lower()]
            if not cp or info is None:
                raise RuntimeError("calibration copy not found in the trace")
            scale[counter] = (info["copy_bytes_read"] / 1024.0) / (sum(cp) / len(cp))
        per = {}
        n_dom = 0
        passes = 4
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            rows, info = run("w_" + counter, counter, ["--workload", workload, "--passes-only", str(link), "--steps", str(passes)] + ([] if TUNE else ["--no-tune"]))
            n = info["kernel_launches_of_the_passes"]
            last = rows[-n:]
            nc = info["n_chains"]
            dom = [i for i, c in enumerate(info["chains"]) if c["kernel"] == "conv3x3_kernel"] or list(range(nc))
            n_dom = len(dom)
            per[counter] = sum(last[p * nc + i][1] for p in range(passes) for i in dom) / passes * 1024.0 * scale[counter]
        total = (per["FETCH_SIZE"] + per["WRITE_SIZE"]) / n_dom
        note = ("measured for this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (one counter per child process) over %d passes of the same "
                "workload, link level and partition policy, scaled by the same counters' reading of a 256 MiB device copy (x %.3f / x %.3f); "
                "fetched %.1f MB + written %.1f MB per launch" % (passes, scale["FETCH_SIZE"], scale["WRITE_SIZE"],
                                                                    per["FETCH_SIZE"] / n_dom / 1e6, per["WRITE_SIZE"] / n_dom / 1e6))
        return total, note
    except Exception as e:      # the profiler is not part of the product: without it the stored summary is quoted instead
        return None, "counter run failed (%s)" % str(e)[:200]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def pmc_traffic(workload):
    """HBM bytes per launch of the dominant kernel.  rocprofv3 counters cannot be read from inside the timed process,
    so this is the value of the committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script
    on the same workload, link level and partition policy), returned with the file it comes from; None if there is none."""
    rel = os.path.join("profiles", "conv3x3_kernel_%s_pmc.txt" % workload)
    val, plan = None, ""
    try:
        for ln in open(os.path.join(ROOT, rel)):
            if ln.startswith("traffic_bytes_per_launch:"):
                val = float(ln.split(":", 1)[1])
            if ln.startswith("plan:"):
                plan = ln.split(":", 1)[1].strip()
    except OSError:
        pass
    if val is None:
        return None, "no counter summary committed for this workload"
    return val, "stored profile value, not measured in this run: %s (%s)" % (rel, plan or "plan not recorded")


TABLE4 = [  # (graph, optimisation the row measures, speed-up the paper prints for it on its DSP)
    ("cbr_maxpool", "linking", 3.3), ("cbr_avgpool", "linking", 2.3), ("fully_connected", "split", 2.25), ("cbr", "split", 2.6)]


def table4_rows(steps, warmup, wg, X, torch):
    """The operator micro-benchmark of Table 4 on this machine: each operator with and without the optimisation its
    row measures (linking: link level 2 vs 1; split: operator split on vs one workgroup), batch 1, bf16."""
    rows = []
    for name, opt, paper in TABLE4:
        g = wg.table4(name, batch=1)
        ms = {}
        for label, link, split in (("with", 2, 1), ("without", 1 if opt == "linking" else 2, 1 if opt == "linking" else 0)):
            s = X.Session(g, link=link, split=split, compute=1)
            s.set_input(g.x)
            ms[label] = time_steps(s, torch, steps, warmup, graph=False)[0]
            s.close()
        rows.append({"operator": name, "optimisation": opt, "ms_with": round(ms["with"], 5), "ms_without": round(ms["without"], 5),
                     "speedup": round(ms["without"] / ms["with"], 2), "paper_speedup_on_its_dsp": paper})
    return rows


def cpu_baseline(g, images):
    """The fp64 oracle as it stands, on `images` images of the same workload, host cores of this machine."""
    from oracle import xenos_oracle as xo
    x = g.x[:images]
    t0 = time.perf_counter()
    xo.forward(g, x)
    dt = time.perf_counter() - t0
    return {"value": images / dt, "unit": "images/s", "cores": xo.threads(), "kind": "oracle",
            "sample": f"{images} of the {g.input_shape[0]} images of the headline batch, full network, fp64, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16_n32_bf16", choices=sorted(WORKLOADS))
    ap.add_argument("--quick", action="store_true", help="headline workload at link levels 3 and 2 only, no CPU baseline, no other workloads")
    ap.add_argument("--cpu-images", type=int, default=0, help="images of the headline batch the oracle is timed on (0 = all)")
    ap.add_argument("--detail", default="", help="write the full per-chain report (JSON) to this file")
    ap.add_argument("--no-tune", action="store_true", help="skip xenos_plan_tune: time the cost model's partition choice")
    ap.add_argument("--passes-only", type=int, default=-1, choices=(-1, 0, 1, 2, 3),
                    help="run the workload at this link level (0 = U0, 1 = U1, 2, 3): tune (unless --no-tune), synchronise, then --steps "
                         "eager passes, and exit: the process whose kernels rocprofv3 traces / counts per link level; the JSON line says "
                         "how many kernel launches the passes are, they are the last ones of the process")
    ap.add_argument("--in-flight", type=int, default=1, choices=(1, 2),
                    help="with --passes-only: passes in flight at a time (2 = the headline's step policy, on two streams)")
    ap.add_argument("--no-traffic", action="store_true", help="do not run the rocprofv3 counter passes that measure roofline.traffic (quote the stored summary)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain device copy of 256 MiB three times and exit (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    global TUNE
    TUNE = not args.no_tune
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    # HBM traffic of the dominant kernel for the roofline: counted by child processes under rocprofv3 while this process has
    # not touched the GPU yet
    live_traffic = (None, "")
    if not (args.quick or args.no_traffic or args.calibrate_copy or args.passes_only >= 0):
        live_traffic = measure_traffic(args.workload, HEADLINE_LINK)

    import torch
    from paper_2302_00282_amd import xenos as X
    from workloads import cnn_graphs as wg
    X.lib()     # fails loudly if the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "copies": 3}))
        return

    name = args.workload
    cfg, batch, compute = WORKLOADS[name]
    stream_note = pick_streams(X, torch)
    if args.passes_only >= 0:
        g = wg.build(cfg, batch)
        s = X.Session(g, link=args.passes_only, split=1, compute=compute)
        s.set_input(g.x)
        retuned = s.tune(reps=5) if TUNE else 0
        torch.cuda.synchronize()
        if args.in_flight == 1:
            for _ in range(args.steps):
                s.run()
        else:
            lane = s.lane()
            lane.x.copy_(s.x)
            streams = _STREAMS[:2]
            torch.cuda.synchronize()
            for k in range(args.steps):
                with torch.cuda.stream(streams[k % 2]):
                    (s.run if k % 2 == 0 else lane.run)()
        torch.cuda.synchronize()
        print(json.dumps({"workload": name, "link": args.passes_only, "passes": args.steps, "passes_in_flight": args.in_flight, "n_chains": s.info["n_chains"],
                          "kernel_launches_of_the_passes": args.steps * s.info["n_chains"], "tuned": bool(TUNE), "chains_retuned": retuned,
                          "algorithmic_hbm_mb_per_pass": s.info["hbm_bytes"] / 1e6,
                          "chains": [dict(name=c["name"], kernel=chain_label(c), gflop=c["flops"] / 1e9,
                                          mb=(c["bytes_in"] + c["bytes_w"] + c["bytes_out"] + c["bytes_res"]) / 1e6) for c in s.info["chains"]]}))
        s.close()
        return
    links = (3, 2) if args.quick else (3, 2, 1, 0)
    head, g = run_workload(name, args.steps, args.warmup, links, chains=True, wg=wg, X=X, torch=torch)
    lk = head[LINK_NAMES[HEADLINE_LINK]]

    # Roofline of the dominant kernel: conv3x3_kernel (halo-staged 3x3 convolution chains on MFMA), over all its
    # launches in one step.  achieved = algorithmic flops of those chains / their summed launch durations, measured
    # with HIP events around every launch on the launch stream.  The other chains are in `per_layer`.
    conv = [c for c in lk["chains"] if c["kind"] == "conv"]
    dom = [c for c in conv if c.get("halo")] or conv
    dom_ms, dom_gf = sum(c["ms"] for c in dom), sum(c["gflop"] for c in dom)
    conv_ms, conv_gf = sum(c["ms"] for c in conv), sum(c["gflop"] for c in conv)
    step_ms = sum(c["ms"] for c in lk["chains"])
    att = attainable(X, torch)
    traffic, traffic_source = live_traffic
    if traffic is None:
        stored, stored_source = pmc_traffic(name)
        traffic, traffic_source = stored, (traffic_source + "; " if traffic_source else "") + stored_source
    roof = {"bound": "mfma", "kernel": "%s (%d launches per step)" % (dom[0]["kernel"], len(dom)),
            "achieved": dom_gf / dom_ms, "peak": PEAK[compute], "unit": "TFLOP/s",
            "frac": dom_gf / dom_ms / PEAK[compute], "traffic": traffic, "traffic_source": traffic_source,
            "avg_launch_ms": dom_ms / len(dom), "avg_launch_ms_between_events": sum(c["ms_between_events"] for c in dom) / len(dom),
            "event_gap_ms_per_launch": lk["event_gap_ms_per_launch"],
            "launch_duration_method": "HIP events around every launch of an instrumented pass, minus the gap the events add per launch "
                                      "= (instrumented pass - plain pass) / launches, both measured in this run",
            "condition": "launch durations of passes that run one at a time: a launch has the chip to itself (the steps behind `value` "
                         "overlap two passes, so a launch there shares the chip and its duration says nothing about the kernel)",
            "flops_per_launch": dom_gf * 1e9 / len(dom),
            "algorithmic_bytes_per_launch": sum(c["mb"] for c in dom) * 1e6 / len(dom),
            "share_of_step": dom_ms / step_ms,
            "attainable_measured_here": {**{k: round(v, 1) for k, v in att.items()},
                                         "frac_of_mfma_loop": dom_gf / dom_ms / att["mfma_loop_tflops_bf16"] if compute == 1 else None,
                                         "frac_of_mfma_loop_relu_like_operands": dom_gf / dom_ms / att["mfma_loop_tflops_bf16_relu_like_operands"] if compute == 1 else None},
            "all_conv_chains": {"n": len(conv), "achieved": conv_gf / conv_ms, "frac": conv_gf / conv_ms / PEAK[compute],
                                "share_of_step": conv_ms / step_ms},
            "best_layer": max(({"name": c["name"], "achieved": c["gflop"] / c["ms"], "frac": c["gflop"] / c["ms"] / PEAK[compute]}
                               for c in dom), key=lambda d: d["achieved"]),
            "per_layer": layer_table(lk["chains"], compute)}
    memb = [r for r in roof["per_layer"] if r["bound"] == "hbm"]
    if memb:    # chains whose arithmetic intensity puts them under the HBM roof (first layer, FC layers, summing passes)
        roof["memory_bound_chains"] = [{"name": r["chain"], "gb_per_s": r["gb_per_s"], "frac_of_hbm": r["frac"],
                                        "frac_of_stream_read": round(r["gb_per_s"] / att["stream_read_gb_per_s"], 4)} for r in memb]

    line = {
        "metric": "images/sec + % MFMA/HBM roofline, linked vs unlinked, batch 1 and 32",
        "value": lk["images_per_s_in_flight"], "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": lk["ms_per_step_in_flight"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": f"config {cfg}: {g.name}-style, batch {batch}, {head['dtype']}, linked+split, "
                               f"synthetic seeded weights and input", "batch": batch, "mode": "linked+split",
                   "link_level": HEADLINE_LINK, "gflop_per_step": head["gflop"], "launch": lk["launch"],
                   "passes_in_flight": IN_FLIGHT, "streams": stream_note,
                   "step_policy": "step k runs on stream k % 2 with that stream's workspace and output (xenos_run / xenos_run_with on one "
                                  "plan): two independent batches are in flight, every step is a whole pass over its own batch",
                   "wall_ms_per_step": lk["wall_ms_per_step_in_flight"],
                   "one_pass_at_a_time": {"ms_per_step": lk["ms_per_step"], "images_per_s": lk["images_per_s"],
                                          "note": "the same steps one after the other on one stream: the latency of a pass, and the "
                                                  "condition under which the roofline of the dominant kernel is measured (a launch "
                                                  "has the chip to itself; the sum of these launch durations is therefore longer than "
                                                  "ms_per_step of the overlapped steps)"},
                   "ms_per_step_graph_replay": lk["ms_per_step_graph_replay"],
                   "ms_per_step_median": lk["ms_per_step_median"], "ms_per_step_min": lk["ms_per_step_min"], "ms_per_step_p90": lk["ms_per_step_p90"],
                   "partition": "profiled per chain (xenos_plan_tune)" if TUNE else "cost model"},
        "tflops": head["gflop"] / lk["ms_per_step_in_flight"],
        "roofline": roof,
        "linked_vs_unlinked": {k: {"images_per_s": head[k]["images_per_s_in_flight"], "ms_per_step": head[k]["ms_per_step_in_flight"],
                                   "images_per_s_one_pass_at_a_time": head[k]["images_per_s"], "ms_per_step_one_pass_at_a_time": head[k]["ms_per_step"],
                                   "n_chains": head[k]["n_chains"], "algorithmic_hbm_mb": head[k]["algorithmic_hbm_mb"]}
                               for k in ("linked_deep", "linked", "U1", "U0") if k in head},
    }
    detail = {"headline": head}
    if not args.quick:
        line["cpu_baseline"] = cpu_baseline(g, batch if args.cpu_images <= 0 else min(args.cpu_images, batch))
        del g
        others = []
        for other in WORKLOADS:
            if other == name:
                continue
            r, _ = run_workload(other, args.steps, args.warmup, (3, 2, 1, 0), chains=True, wg=wg, X=X, torch=torch)
            detail[other] = r
            d3 = r["linked_deep"]
            ocomp = WORKLOADS[other][2]
            rows = layer_table(d3["chains"], ocomp)
            worst = min(rows, key=lambda x: x["frac"])
            others.append({"workload": other, "gflop": round(r["gflop"], 3), "passes_timed": r["passes_timed"],
                           **{k: round(r[k]["images_per_s"], 1) for k in ("linked_deep", "linked", "U1", "U0") if k in r},
                           "linked_deep_graph_replay": round(d3["images_per_s_graph_replay"], 1),
                           "linked_deep_two_passes_in_flight": round(d3["images_per_s_in_flight"], 1),
                           "ms_per_step_two_passes_in_flight": round(d3["ms_per_step_in_flight"], 4),
                           "ms_per_step": round(d3["ms_per_step"], 4), "ms_per_step_median": round(d3["ms_per_step_median"], 4), "n_chains": d3["n_chains"],
                           "tflops": round(d3["tflops"], 2), "frac_of_mfma_peak": round(d3["tflops"] / PEAK[ocomp], 4),
                           "algorithmic_hbm_mb": round(d3["algorithmic_hbm_mb"], 2),
                           "algorithmic_gb_per_s": round(d3["algorithmic_gb_per_s"], 1),
                           "frac_of_hbm_peak": round(d3["algorithmic_gb_per_s"] / HBM_PEAK, 4),
                           "unlinked_U0_hbm_mb": round(r["U0"]["algorithmic_hbm_mb"], 2),
                           "slowest_chain_vs_its_roof": {"chain": worst["chain"], "kernel": worst["kernel"], "bound": worst["bound"], "frac": worst["frac"]}})
        line["other_workloads"] = others
        line["table4_micro_benchmark"] = table4_rows(max(args.steps, 50), args.warmup, wg, X, torch)
    if args.detail:
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(detail, f, indent=1)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
