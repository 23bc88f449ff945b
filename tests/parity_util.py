"""Helpers of the GPU parity tests: error metric, bf16 rounding in integer arithmetic, an on-disk cache of oracle
outputs, the oracle run on bf16-pre-rounded operands, and teacher-forced per-chain parity.

Nothing here computes the method: the oracle (oracle/) supplies every expected value, the HIP library
(through its C ABI) every measured one.
"""
import copy
import hashlib
import os
import tempfile

import numpy as np

from oracle import xenos_oracle as xo

TOL = {0: 1e-5, 1: 2e-2}          # XENOS_F32, XENOS_BF16: max|gpu - ref| / max|ref|, the end-to-end bars
# One chain fed the oracle's own activation (rounded to the storage type) and compared with the oracle's result for
# those same inputs: what is left is the fp32 accumulation order (the fp32 bar, 1e-5 of max|ref|, covers it) and, on the
# bf16 path, ONE rounding of each output element to bf16, i.e. at most half a bf16 ulp OF THAT ELEMENT (8 significant
# bits: 2^(e-8) for |ref| in [2^e, 2^(e+1))).  The bf16 bar is therefore element-wise:
#   |gpu - ref| <= half_ulp_bf16(ref) + 2e-5 * max|ref|      (chain_excess <= 1)
# which a wrong tap, index or weight fails on any element it touches, small ones included.  Chains that keep a
# bf16-rounded intermediate on chip (two operators in one kernel) carry the propagated rounding of that intermediate,
# which is not proportional to the output element: they are held to 6e-3 of max|ref| (measured: up to 4.6e-3).
TOL_CHAIN = {0: 1e-5, 1: 4e-3}
TOL_CHAIN_TWO_ROUNDINGS = 6e-3


def chain_excess(got, ref):
    """max over elements of |got - ref| / (half a bf16 ulp of ref + 2e-5 max|ref|): <= 1 for a correctly rounded result."""
    ref = np.asarray(ref, np.float64)
    a = np.abs(ref)
    e = np.floor(np.log2(np.maximum(a, 1e-300)))
    half_ulp = np.where(a > 0, np.exp2(e - 8), 0.0)
    bound = half_ulp + 2e-5 * max(a.max(), 1e-30)
    return float((np.abs(got.astype(np.float64) - ref) / bound).max())


def rel_err(y, ref, scale=None):
    s = max(np.abs(ref).max(), 1e-30) if scale is None else scale
    return float(np.abs(y.astype(np.float64) - ref).max() / s)


def bf16_rne(x):
    """fp32 -> bf16 -> fp32 with round-to-nearest-even, in integer arithmetic."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32)


def bf16_bits(x):
    """fp32 array -> uint16 array of bf16 bit patterns (round-to-nearest-even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------------------------------------- oracle cache
def _cache_dir():
    d = os.environ.get("XENOS_ORACLE_CACHE") or os.path.join(tempfile.gettempdir(), "xenos_oracle_cache")
    os.makedirs(d, exist_ok=True)
    return d


def cached_forward(g, tag):
    """xo.forward(g) for a full-size configuration, kept on disk keyed by (tag, graph name, input shape, a digest of the
    seeded input), so that several tests and link levels of one run pay for the oracle once."""
    h = hashlib.sha1(np.ascontiguousarray(g.x).view(np.uint8)[:1 << 20].tobytes()).hexdigest()[:16]
    path = os.path.join(_cache_dir(), "%s_%s_%s_%s.npy" % (tag, g.name, "x".join(map(str, g.input_shape)), h))
    if os.path.exists(path):
        return np.load(path)
    ref = xo.forward(g)
    np.save(path, ref)
    return ref


# ---------------------------------------------------------------------------------------------- bf16 diagnostic oracle
def rounded_graph(g):
    """The same graph with its input and its conv / fc / matmul weights pre-rounded to bf16 (RNE), still fp32 arrays: the
    oracle then computes, in fp64, what the bf16 path would compute with exact arithmetic and exact intermediates,
    which separates kernel error from the quantisation of the operands.  Biases and BN parameters stay fp32 (the
    library folds them in fp64 and applies them to the fp32 accumulator)."""
    g2 = copy.copy(g)
    g2.x = bf16_rne(g.x)
    g2.ops = []
    for op in g.ops:
        o = copy.copy(op)
        if op.kind in ("conv", "fc", "matmul"):
            o.params = dict(op.params)
            o.params["weight"] = bf16_rne(op.params["weight"])
        g2.ops.append(o)
    return g2


def last_chain_scale(g, acts):
    """max |value| over the output of the last conv / fc operator and everything computed from it: the scale of the
    last chain before its activations and reductions.  A graph output of a handful of values that are sums with
    cancellation can be far smaller than the numbers it was computed from; an error bound relative to max|output|
    alone then measures that cancellation, not the kernels."""
    last = max((i for i, op in enumerate(g.ops) if op.kind in ("conv", "fc")), default=0)
    return max(float(np.abs(acts[t]).max()) for t in range(last + 1, len(g.ops) + 1) if t in acts)


# ---------------------------------------------------------------------------------------------- teacher forcing
def _view_tensor(acts, v):
    """The oracle's value of what view `v` of the plan holds: channels c0, c0 + cs, ... of graph tensor v['tensor']."""
    t = acts[v["tensor"]]
    idx = v["c0"] + v["cs"] * np.arange(v["c"])
    a = t[:, idx]
    assert a.shape == (v["n"], v["c"], v["h"], v["w"]), (a.shape, v)
    return a


def _index(v):
    """Element offsets (in elements of the view's type, from its byte_off) of the view's (n, c, h, w) elements."""
    n, c, h, w = v["n"], v["c"], v["h"], v["w"]
    return (np.arange(n)[:, None, None] * v["sN"] + np.arange(c)[None, :, None] * v["sK"] +
            np.arange(h * w)[None, None, :] * v["sP"]).reshape(n, c, h, w)


def _mem(sess, v):
    torch = sess.torch
    if v["mem"] == "workspace":
        return sess.workspace_view()
    t = sess.x if v["mem"] == "input" else sess.y
    return t.view(-1).view(torch.uint8)


def write_view(sess, v, a):
    """Stores the fp64 array `a` (n, c, h, w) into view `v`, rounded to the view's element type."""
    torch = sess.torch
    mem = _mem(sess, v)
    idx = torch.from_numpy(_index(v).reshape(-1)).to(sess.device)
    lo = v["byte_off"]
    if v["esz"] == 4:
        flat = mem[lo:lo + (int(idx.max()) + 1) * 4].view(torch.float32)
        flat[idx] = torch.from_numpy(a.astype(np.float32).reshape(-1)).to(sess.device)
    else:
        flat = mem[lo:lo + (int(idx.max()) + 1) * 2].view(torch.int16)
        flat[idx] = torch.from_numpy(bf16_bits(a.astype(np.float32)).view(np.int16).reshape(-1)).to(sess.device)


def read_view(sess, v):
    torch = sess.torch
    mem = _mem(sess, v)
    idx = torch.from_numpy(_index(v).reshape(-1)).to(sess.device)
    lo = v["byte_off"]
    if v["esz"] == 4:
        out = mem[lo:lo + (int(idx.max()) + 1) * 4].view(torch.float32)[idx].cpu().numpy()
    else:
        bits = mem[lo:lo + (int(idx.max()) + 1) * 2].view(torch.int16)[idx].cpu().numpy().view(np.uint16)
        out = bits_to_f32(bits)
    return out.reshape(v["n"], v["c"], v["h"], v["w"])


def _storage_round(a, v):
    """`a` as the view's element type holds it (bf16 views: rounded to nearest even), back in fp64."""
    return (bf16_rne(a.astype(np.float32)) if v["esz"] == 2 else a.astype(np.float32)).astype(np.float64)


_MOVES = ("concat", "slice", "shuffle")


def _chain_reference(g, ch, v, acts, forced, rnd):
    """What the oracle computes for output view `v` of chain `ch` from the inputs the chain was given: the chain's
    operators, in graph order, applied to `forced` (graph tensor id -> the stored, rounded value written to the device)
    for tensors that come from outside the chain."""
    ops = sorted(set(ch["ops"]))
    if not ops or all(g.ops[o].kind in _MOVES for o in ops):
        # pure data movement (a copied concat part, a strided shuffle copy, the import pass): the view's tensor, as stored
        return _storage_round(_view_tensor(acts, v), v)
    shapes = g.shapes()
    vals, parts = {}, {}
    for o in ops:
        op = g.ops[o]
        if op.kind in _MOVES:
            continue
        t0 = op.inputs[0]
        if (op.kind in ("maxpool", "avgpool", "gap") and t0 not in vals and t0 >= 1 and g.ops[t0 - 1].kind == "concat"
                and any(t in vals for t in g.ops[t0 - 1].inputs)):
            # a pooling that the plan moved in front of the concat it follows: it pools this chain's part(s) of the concat
            off = 0
            for t in g.ops[t0 - 1].inputs:
                if t in vals:
                    parts[(o + 1, off)] = xo.apply_op(op, [vals[t]])
                off += shapes[t][1]
            continue
        # (a tensor the chain reads through another view, e.g. behind a shuffle folded into its weights, holds the same
        # stored values)
        ins = [vals[t] if t in vals else forced[t] if t in forced else rnd(acts[t]) for t in op.inputs]
        vals[o + 1] = xo.apply_op(op, ins)
    key = (v["tensor"], v["c0"])
    if key in parts and parts[key].shape[1] == v["c"]:
        return parts[key]
    r = vals[v["tensor"]] if v["tensor"] in vals else vals[max(vals)]
    if r.shape[1] == v["c"]:
        return r                                      # the chain's tensor itself
    pos = ch.get("shuffle_store", 0)
    if pos:
        # the chain stores its channels and those of the other part of its concat, alternating (two-group shuffle)
        full = _storage_round(_view_tensor(acts, v), v)
        full[:, (pos - 1)::2] = r
        return full
    return r[:, v["c0"] + v["cs"] * np.arange(v["c"])]


def teacher_forced(g, sess, compute, acts=None):
    """Per-chain parity with every chain fed the oracle's activations, so that one bad layer cannot hide under an
    end-to-end budget.  `sess` is a bound Session of `g` whose full pass has run once (so that padding channels and
    slack hold finite values).  For every step of the plan, in order: its inputs that are graph tensors are
    overwritten with the oracle's values rounded to the storage type, the step alone is launched through
    xenos_run_chain, and its output, where it is a graph tensor, is compared with what the oracle computes for the
    chain's operators FROM THOSE SAME ROUNDED INPUTS (the oracle runs on bf16-pre-rounded weights on the bf16 path).
    What is left is the kernel's own error: accumulation order and one rounding of the output to the storage type.
    Returns [(chain name, kernel label, rel err of max|ref|, chain_excess (bf16 outputs) or 0)]."""
    torch = sess.torch
    g2 = rounded_graph(g) if compute == 1 else g
    if acts is None:
        acts = xo.run_graph(g2, keep="all")
    rows = []
    forced, pending = {}, ""
    rnd = (lambda a: bf16_rne(a.astype(np.float32)).astype(np.float64)) if compute == 1 else (lambda a: a.astype(np.float32).astype(np.float64))
    for ch in sess.info["chains"]:
        if ch["in"]["tensor"] >= 0:
            forced = {}                               # (the summing pass of a reduction split keeps its chain's inputs)
        for key in ("in", "in2"):
            v = ch.get(key)
            if v is not None and v["tensor"] >= 0 and v["mem"] != "output":
                want = _view_tensor(acts, v)
                write_view(sess, v, want)
                full = _storage_round(acts[v["tensor"]], v)
                forced[v["tensor"]] = full
        sess.run_chain(ch["i"])
        torch.cuda.synchronize()
        v = ch["out"]
        label = ch["kind"]
        if ch["kind"] == "conv":
            label = "halo" if ch.get("halo") else ch.get("loader", "conv")
            if ch.get("dw_linked") and label not in ("stem", "pair", "pwdw"):
                label = "dw+" + label
        elif ch["kind"] == "splitk_finish":
            label = pending + ".sum"                  # the summing pass completes the chain of the step before it
        pending = label
        if v["tensor"] < 0:
            continue                                  # partial sums of a reduction split: finished by the next step
        if ch.get("out2") is not None:                # a chain with two outputs (the two expand parts of a Fire module)
            v2 = ch["out2"]
            rows.append((ch["name"] + ".out2", label, rel_err(read_view(sess, v2), _chain_reference(g2, ch, v2, acts, forced, rnd)), 0.0))
        ref = _chain_reference(g2, ch, v, acts, forced, rnd)
        got = read_view(sess, v)
        rows.append((ch["name"], label, rel_err(got, ref), chain_excess(got, ref) if v["esz"] == 2 else 0.0))
    return rows
