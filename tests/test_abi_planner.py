"""CPU-side checks (no GPU): the C-ABI library loads and exports every symbol the header declares,
graph ingest validates and infers shapes, and the optimiser (fusion pre-pass, operator linking,
operator split) produces plans that are structurally sound.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2302_00282_amd import xenos as X
from workloads import cnn_graphs as wg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def plan_json(g, **kw):
    G = X.graph_from_workload(g)
    try:
        P = X.xenos_plan_link_split(G, **kw)
        try:
            return X.xenos_plan_query(P)
        finally:
            X.xenos_destroy(P)
    finally:
        X.xenos_destroy(G)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "xenos.h")).read()
    names = set(re.findall(r"\b(xenos_[a-z_]+)\s*\(", hdr))
    assert {"xenos_graph_create", "xenos_plan_link_split", "xenos_run", "xenos_destroy"} <= names
    lib = ctypes.CDLL(X.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(X, "_lib", None)
    monkeypatch.setattr(X, "LIB_PATH", "/nonexistent/libxenos.so")
    with pytest.raises(ImportError):
        X.lib()


def test_graph_validation_errors():
    g = wg.single_chain(batch=1)
    keep = []
    ops = X.op_descs(g, keep)
    ind = X.TensorDesc(1, 3, 32, 32, X.XENOS_F32, X.XENOS_NCHW)
    with pytest.raises(X.XenosError) as e:
        X.xenos_graph_create(ind, ops, 9)                      # output id out of range
    assert e.value.status == X.XENOS_EINVAL
    bad = X.op_descs(g, keep)
    bad[0].weight = ctypes.cast(None, ctypes.POINTER(ctypes.c_float))
    with pytest.raises(X.XenosError) as e:
        X.xenos_graph_create(ind, bad, 4)
    assert e.value.status == X.XENOS_EINVAL and "weight" in str(e.value)
    bad = X.op_descs(g, keep)
    bad[0].kh = bad[0].kw = 40                                 # kernel larger than the padded map
    with pytest.raises(X.XenosError) as e:
        X.xenos_graph_create(ind, bad, 4)
    assert e.value.status == X.XENOS_ESHAPE
    with pytest.raises(X.XenosError) as e:                     # wrong output descriptor
        X.xenos_graph_create(ind, ops, 4, X.TensorDesc(1, 16, 8, 8, X.XENOS_F32, X.XENOS_NCHW))
    assert e.value.status == X.XENOS_ESHAPE
    b = wg.builder("bad_add", (1, 8, 8, 8), 1)
    t1 = b.conv(0, 8, 3, 1, 1)
    t2 = b.conv(0, 8, 3, 2, 1)
    b.g.ops.append(wg.Op("add", [t1, t2]))
    with pytest.raises(X.XenosError) as e:
        X.xenos_graph_create(X.TensorDesc(1, 8, 8, 8, 0, 0), X.op_descs(b.g, keep), 3)
    assert e.value.status == X.XENOS_ESHAPE
    assert X.xenos_destroy(None) is None


def test_slice_and_shuffle_validation():
    g = wg.single_chain(batch=1)                                   # 16 output channels
    g.ops.append(wg.Op("slice", [len(g.ops)], dict(c_begin=10, out_c=8), {}, "s"))
    g.output = len(g.ops)
    with pytest.raises(X.XenosError) as e:
        X.graph_from_workload(g)
    assert e.value.status == X.XENOS_ESHAPE and "slice" in str(e.value)
    g.ops[-1] = wg.Op("shuffle", [len(g.ops) - 1], dict(groups=3), {}, "s")
    with pytest.raises(X.XenosError) as e:
        X.graph_from_workload(g)
    assert e.value.status == X.XENOS_ESHAPE and "shuffle" in str(e.value)
    g.ops[-1] = wg.Op("shuffle", [len(g.ops) - 1], dict(groups=4), {}, "s")
    j = plan_json(g, link=2)["plan"]
    assert j["linked_shuffles"] == 0 and sum(1 for c in j["chains"] if c["kind"] == "elt") == 4   # one strided copy per group


def test_plan_option_errors():
    G = X.graph_from_workload(wg.single_chain(batch=1))
    try:
        with pytest.raises(X.XenosError):
            X.xenos_plan_link_split(G, link=7)
        with pytest.raises(X.XenosError):
            X.xenos_plan_link_split(G, hw=dict(num_cu=0, lds_bytes_per_cu=0, l2_bytes=0, llc_bytes=0, hbm_bytes=0))
        with pytest.raises(X.XenosError) as e:                 # private memory too small for any parameter split
            X.xenos_plan_link_split(G, hw=dict(num_cu=8, lds_bytes_per_cu=4096, l2_bytes=0, llc_bytes=0, hbm_bytes=0))
        assert e.value.status == X.XENOS_EUNSUPPORTED
    finally:
        X.xenos_destroy(G)


def test_cfg0_links_to_one_chain_and_unlinked_levels():
    g = wg.build(0, 1)
    q2 = plan_json(g, link=2)["plan"]
    q1 = plan_json(g, link=1)["plan"]
    q0 = plan_json(g, link=0)["plan"]
    assert q2["n_chains"] == 1 and q2["chains"][0]["ops"] == [0, 1, 2, 3]       # CBR + MaxPool = one pass (CBRM)
    assert q2["chains"][0]["mode"] == "zigzag"
    assert [c["ops"] for c in q1["chains"] if c["kind"] == "conv"] == [[0, 1, 2]]   # fused CBR, pool separate
    assert sum(1 for c in q0["chains"] if c["ops"]) == 4                            # operator by operator
    assert q0["hbm_bytes"] > q1["hbm_bytes"] > q2["hbm_bytes"]


@pytest.mark.parametrize("cfg,batch", [(1, 1), (2, 1), (2, 32), (4, 1), (4, 32)])
def test_every_operator_runs_exactly_once(cfg, batch):
    g = wg.build(cfg, batch, draw=False)
    for link in (0, 1, 2):
        q = plan_json(g, link=link, compute=X.XENOS_BF16)["plan"]
        # (the summing pass of a reduction split completes the chain of the step before it and names the same operators)
        seen = [o for c in q["chains"] if c["kind"] != "splitk_finish" for o in c["ops"]]
        # a hoisted pooling operator appears once per concat producer; a copied concat once per input
        assert set(seen) == set(range(len(g.ops))) - ({i for i, o in enumerate(g.ops) if o.kind == "concat"} if link >= 2 else set())
        if link < 2:
            non_cat = [o for o in seen if g.ops[o].kind != "concat"]
            assert len(non_cat) == len(set(non_cat))


def test_linking_patterns_of_the_workloads():
    g2 = wg.build(2, 1, draw=False)
    res = plan_json(g2, link=2, compute=X.XENOS_BF16)["plan"]
    convs = [c for c in res["chains"] if c["kind"] == "conv"]
    # every shortcut add is executed by a conv chain (in its epilogue, or in the summing pass of a reduction split)
    assert sum(any(g2.ops[o].kind == "add" for o in c["ops"]) for c in convs) == 8
    # the 7x7/2 first layer reads the caller's NCHW tensor in place with its 3x3/2 max-pool linked (CBRM): no pass of its own
    assert convs[0]["loader"] == "stem" and any(g2.ops[o].kind == "maxpool" for o in convs[0]["ops"]) and convs[0]["pool"] != 0
    assert all(c["kind"] in ("conv", "splitk_finish") for c in res["chains"])
    # (on the fp32 path the first layer gathers from memory and its pooling is the only stand-alone pass)
    r32 = plan_json(g2, link=2, compute=X.XENOS_F32)["plan"]
    assert r32["chains"][0]["loader"] == "stem" and r32["chains"][1]["kind"] == "pool"
    assert all(c["kind"] in ("conv", "splitk_finish") for c in r32["chains"][2:])
    # last block + global average (CBRA): through the summing pass of a reduction split (batch 1: the gather kernel's
    # split, batch 32: channel chunks shared out inside the halo-staged kernel); without the operator split the average
    # runs in the convolution's own epilogue.  Either way it is an operator of that chain, not a pass of its own
    assert any(g2.ops[o].kind == "gap" for o in convs[-2]["ops"]) and convs[-2]["mode"] == "flat"
    assert res["chains"][convs[-2]["i"] + 1]["kind"] == "splitk_finish"
    res32 = plan_json(wg.build(2, 32, draw=False), link=2, compute=X.XENOS_BF16)["plan"]
    last32 = [c for c in res32["chains"] if c["kind"] == "conv"][-2]
    assert last32["mode"] == "flat" and last32["halo"] == 1 and last32["ksplit"] > 1 and any(g2.ops[o].kind == "gap" for o in last32["ops"])
    assert res32["chains"][last32["i"] + 1]["kind"] == "splitk_finish"
    # the 7x7 x 512 layers at batch 32: 9 pixel tiles x 4 channel tiles would occupy 36 of 256 units; their channel
    # chunks are shared out so that at least half the units work
    shared = [c for c in res32["chains"] if c["kind"] == "conv" and c["halo"] == 1 and c["ksplit"] > 1]
    assert len(shared) == 3 and all(c["H"] == 7 and 2 * c["tiles_m"] * c["tiles_n"] * c["ksplit"] >= 256 for c in shared)
    u32 = plan_json(wg.build(2, 32, draw=False), link=2, split=0, compute=X.XENOS_BF16)["plan"]
    assert [c for c in u32["chains"] if c["kind"] == "conv"][-2]["mode"] == "gap"
    assert not any(c["kind"] == "splitk_finish" for c in u32["chains"])
    sq = plan_json(wg.build(4, 1, draw=False), link=2, compute=X.XENOS_BF16)["plan"]
    # bf16: the 3x3/2 first layer stages its input block in LDS and its 3x3/2 ceil-mode pool is linked into it; fp32: the
    # gather form of the first-layer kernel, then the pool as the only stand-alone pass
    assert sq["chains"][0]["loader"] == "stem" and sq["chains"][0]["pool"] != 0
    assert all(c["kind"] in ("conv", "splitk_finish") for c in sq["chains"])   # concat and the pools cost no pass
    assert sum(c.get("mode") == "patch" for c in sq["chains"][1:]) == 4      # 3x3/2 ceil-mode pools linked into both expand convs, twice
    sq32 = plan_json(wg.build(4, 1, draw=False), link=2, compute=X.XENOS_F32)["plan"]
    assert sq32["chains"][0]["loader"] == "stem" and sq32["chains"][1]["kind"] == "pool"
    assert all(c["kind"] in ("conv", "splitk_finish") for c in sq32["chains"][2:])
    # a first layer of 24 channels (ShuffleNet-style graph) runs on the same kernel, padded to 32
    sh = plan_json(wg.shufflenet_v2(batch=1, draw=False), link=2, compute=X.XENOS_BF16)["plan"]
    assert sh["chains"][0]["loader"] == "stem" and sh["chains"][0]["K"] == 32 and sh["chains"][0]["pool"] != 0
    offs = sorted({(c["out_c_off"], c["out_sP"]) for c in sq["chains"] if c["kind"] == "conv" and c["out_c_off"]})
    assert (64, 128) in offs and (256, 512) in offs            # expand3x3 halves land at their channel offset
    vgg = plan_json(wg.build(3, 2, draw=False), link=2, compute=X.XENOS_BF16)["plan"]
    assert [c["mode"] for c in vgg["chains"] if c["kind"] == "conv"].count("zigzag") == 5
    # the layout transform of the graph input is linked into the first layer: no import pass, the caller's NCHW
    # tensor is read where it lies; un-linked plans convert first
    assert vgg["chains"][0]["kind"] == "conv" and vgg["chains"][0]["loader"] == "stem"
    vgg1 = plan_json(wg.build(3, 2, draw=False), link=1, compute=X.XENOS_BF16)["plan"]
    assert vgg1["chains"][0]["name"] == "import" and vgg1["chains"][1]["loader"] == "vector"


def test_shufflenet_units_link_their_shuffles():
    # ShuffleNet (Section 7.1): every unit ends in concat -> channel shuffle.  Linked, the shuffle is the order in which
    # the concat's parts are stored: no pass of its own.  The last chain of a unit reads the other half (the pass-through
    # half, or the other branch of a down-sampling unit) in its epilogue and stores both, alternating: no copy either.
    g = wg.shufflenet_v2(batch=1, draw=False)
    n_shuffle = sum(1 for op in g.ops if op.kind == "shuffle")
    assert n_shuffle == 16
    plans = {link: plan_json(g, link=link, compute=1)["plan"] for link in (0, 1, 2, 3)}
    for link in (2, 3):
        j = plans[link]
        assert j["linked_shuffles"] == n_shuffle
        assert sum(1 for c in j["chains"] if c["kind"] == "elt") == 0
        assert sum(1 for c in j["chains"] if c.get("shuffle_store")) == n_shuffle
        ran = sorted(o for c in j["chains"] for o in c["ops"])
        gone = {i for i, op in enumerate(g.ops) if op.kind in ("shuffle", "slice")}    # views and store orders: no pass
        cats = {i for i, op in enumerate(g.ops) if op.kind == "concat"}
        assert set(ran) | gone | cats == set(range(len(g.ops))) and not (set(ran) & {i for i in gone if g.ops[i].kind == "shuffle"})
    for link in (0, 1):
        j = plans[link]
        assert j["linked_shuffles"] == 0
        # un-linked: concat copies both parts, the shuffle copies both groups
        assert sum(1 for c in j["chains"] if c["kind"] == "elt" and "group" in c["name"]) == 2 * n_shuffle
    assert plans[2]["hbm_bytes"] < plans[1]["hbm_bytes"] < plans[0]["hbm_bytes"]
    assert plans[2]["n_chains"] < plans[1]["n_chains"] < plans[0]["n_chains"]


@pytest.mark.parametrize("cfg,batch,compute", [(1, 1, 0), (2, 32, 1), (3, 32, 1), (4, 32, 0)])
def test_split_covers_the_output_and_fits_private_memory(cfg, batch, compute):
    g = wg.build(cfg, batch, draw=False)
    q = plan_json(g, link=2, compute=compute)
    for c in q["plan"]["chains"]:
        if c["kind"] != "conv":
            continue
        assert c["lds"] <= X.MI355X["lds_bytes_per_cu"]
        assert c["tiles_n"] * c["bn"] >= c["K"] > (c["tiles_n"] - 1) * c["bn"]      # outC partition, no gap, no overlap
        if c.get("halo"):
            # halo-staged kernel: TH x TW tiles over the images stacked with their two padding rows each
            assert c["th"] * c["tw"] <= c["bm"] == 256
            assert c["tiles_m"] == -(-(c["N"] * (c["H"] + 2)) // c["th"]) * -(-c["W"] // c["tw"])
        elif c["loader"] == "stem" and c["bm"] == 128:
            # first layer with its input block staged on chip: 8 x 16 tiles of output pixels (3 x 8 pooling windows) per image
            if c["pool"]:
                assert c["tiles_m"] == c["N"] * -(-c["PH"] // 3) * -(-c["PW"] // 8)
            else:
                assert c["tiles_m"] == c["N"] * -(-c["OH"] // 8) * -(-c["OW"] // 16)
        elif c["mode"] == "flat":
            m = c["N"] * c["OH"] * c["OW"]
            assert c["tiles_m"] * c["bm"] >= m > (c["tiles_m"] - 1) * c["bm"]
        elif c["mode"] == "zigzag":
            m = c["N"] * c["PH"] * c["PW"] * 4
            assert c["tiles_m"] * c["bm"] >= m > (c["tiles_m"] - 1) * c["bm"]
        elif c["mode"] == "patch":
            assert c["patch_h"] * c["patch_w"] <= c["bm"]
            py, px = -(-c["PH"] // c["pph"]), -(-c["PW"] // c["ppw"])
            assert c["tiles_m"] == c["N"] * py * px
        if c.get("halo"):
            assert 1 <= c["grid"] <= max(8, X.MI355X["num_cu"])      # persistent workgroups walk the tiles
        elif c["loader"] == "stem" and c["bm"] == 128:
            assert c["tiles_n"] == 1 and 1 <= c["grid"] <= c["tiles_m"]                               # persistent workgroups walk the tiles
        elif c["loader"] == "stem":
            assert c["bm"] == 32 and c["tiles_n"] == 1 and 1 <= c["grid"] <= -(-c["tiles_m"] // 4)   # wavefronts stride over 32-pixel blocks
        else:
            assert c["grid"] >= c["tiles_m"] * c["tiles_n"]
    assert q["workspace_bytes"] > 0 and q["weight_bytes"] > 0


def test_unsplit_plan_uses_one_workgroup():
    q = plan_json(wg.build(0, 1), link=2, split=0)["plan"]
    assert all(c["grid"] == 1 for c in q["chains"] if c["kind"] == "conv")


def test_hardware_description_drives_the_split():
    g = wg.build(2, 32, draw=False)
    big = plan_json(g, compute=1)["plan"]
    small = plan_json(g, compute=1, hw=dict(num_cu=8, lds_bytes_per_cu=160 * 1024, l2_bytes=1 << 20, llc_bytes=0, hbm_bytes=1 << 30))["plan"]
    tb = sum(c["tiles_m"] * c["tiles_n"] for c in big["chains"] if c["kind"] == "conv")
    ts = sum(c["tiles_m"] * c["tiles_n"] for c in small["chains"] if c["kind"] == "conv")
    assert ts <= tb            # fewer units -> never a finer split


def test_planning_time_is_reported_scale():
    import time
    g = wg.build(1, 1)
    G = X.graph_from_workload(g)
    t0 = time.perf_counter()
    P = X.xenos_plan_link_split(G, compute=X.XENOS_BF16)
    dt = time.perf_counter() - t0
    X.xenos_destroy(P)
    X.xenos_destroy(G)
    assert dt < 5.0            # the paper reports 0.11 s for MobileNet (Table 2); same order of magnitude


def test_table4_graphs_follow_the_printed_shapes():
    # tests/golden/table4_shapes.txt holds the shapes printed in Table 4 (first row with the stated reading)
    import os
    rows = {}
    for ln in open(os.path.join(os.path.dirname(__file__), "golden", "table4_shapes.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        f = ln.split()
        rows[f[0]] = [int(x) for x in f[1:8]]
    names = {"cbr_maxpool": "CBR-MaxPooling", "cbr_avgpool": "CBR-AvgPooling", "fully_connected": "FullyConnected", "cbr": "CBR"}
    assert set(names) == set(wg.TABLE4)
    for key, printed in names.items():
        h, w, c, r, s_, c2, k = rows[printed]
        assert wg.TABLE4[key][:6] == (h, w, c, r, s_, k) and c2 == c
        g = wg.table4(key, batch=1, draw=False)
        q = plan_json(g, link=2, compute=X.XENOS_BF16)["plan"]
        assert sum(ch["kind"] == "conv" for ch in q["chains"]) == 1                  # one linked chain each (plus the input conversion)
        assert all(ch["kind"] in ("conv", "cvt", "splitk_finish") for ch in q["chains"])


def test_partition_candidates_and_tune_argument_checks():
    # every convolution chain carries the legal partitions the split planner found (what xenos_plan_tune profiles);
    # chains whose plan structure depends on the choice carry none
    q = plan_json(wg.build(3, 32, draw=False), link=2, compute=X.XENOS_BF16)["plan"]
    convs = [c for c in q["chains"] if c["kind"] == "conv"]
    assert convs[0]["loader"] == "stem" and convs[0]["candidates"] == 0
    assert all(c["candidates"] >= 3 for c in convs[1:13])              # general tiles + halo tiles for the 3x3 layers
    assert all(c["candidates"] == 0 for c in convs if c["ksplit"] > 1)
    assert all(c["tuned"] == 0 for c in convs)
    forced = plan_json(wg.build(0, 1), link=2, tile=3)["plan"]
    assert all(c["candidates"] == 0 for c in forced["chains"] if c["kind"] == "conv")
    G = X.graph_from_workload(wg.build(0, 1))
    P = X.xenos_plan_link_split(G)
    try:
        with pytest.raises(X.XenosError) as e:
            X.xenos_plan_tune(P, 256, 256)                             # not bound: rejected before anything is launched
        assert e.value.status == X.XENOS_EINVAL
        with pytest.raises(X.XenosError):
            X.xenos_plan_tune(P, 0, 256)
    finally:
        X.xenos_destroy(P)
        X.xenos_destroy(G)


def test_run_entry_points_reject_bad_arguments_before_any_launch():
    # xenos_run / xenos_run_with / xenos_run_static / xenos_run_graph / xenos_run_chain on a plan that is not bound, and
    # null pointers: XENOS_EINVAL with a message, nothing touches the device (there is none here)
    G = X.graph_from_workload(wg.build(0, 1))
    P = X.xenos_plan_link_split(G)
    try:
        for call in (lambda: X.xenos_run(P, 256, 256), lambda: X.xenos_run_with(P, 256, 256, 256), lambda: X.xenos_run_static(P, 256, 256),
                     lambda: X.xenos_run_graph(P, 256, 256), lambda: X.xenos_run_chain(P, 0, 256, 256)):
            with pytest.raises(X.XenosError) as e:
                call()
            assert e.value.status == X.XENOS_EINVAL and "bound" in str(e.value)
        for call in (lambda: X.xenos_run_with(P, 0, 256, 256), lambda: X.xenos_run_with(P, 256, 0, 256), lambda: X.xenos_run_with(P, 256, 256, 0),
                     lambda: X.xenos_run(P, 0, 256)):
            with pytest.raises(X.XenosError) as e:
                call()
            assert e.value.status == X.XENOS_EINVAL
    finally:
        X.xenos_destroy(P)
        X.xenos_destroy(G)


# ------------------------------------------------------------------------------------------ link level 3, one test per pattern
def _kinds(g, c):
    return [g.ops[o].kind for o in c["ops"]]


def test_pattern_pointwise_to_depthwise_on_chip():
    # Section 2.2 / Table 1 (ConvX -> ConvY): a depthwise-separable stack becomes pointwise -> depthwise chains, the
    # tensors that reach memory are the (smaller) depthwise outputs
    g = wg.build(1, 1, draw=False)
    for compute in (X.XENOS_BF16, X.XENOS_F32):
        l2 = plan_json(g, link=2, compute=compute)["plan"]
        l3 = plan_json(g, link=3, compute=compute)["plan"]
        pw = [c for c in l3["chains"] if c.get("loader") == "pwdw"]
        assert len(pw) == 12 and l3["n_chains"] <= l2["n_chains"] - 12
        for c in pw:
            assert _kinds(g, c) == ["conv", "bn", "relu", "conv", "bn", "relu"]
            conv1, conv2 = [o for o in c["ops"] if g.ops[o].kind == "conv"]
            assert g.ops[conv1].attrs["groups"] == 1 and g.ops[conv2].attrs["groups"] == c["K"]
            s = g.ops[conv2].attrs["stride"]
            # tiles of depthwise output pixels cover the output; the staged block of the pointwise output fits the kernel's LDS block
            assert c["tiles_m"] == c["N"] * -(-c["OH"] // c["th"]) * -(-c["OW"] // c["tw"]) and c["tiles_n"] == -(-c["K"] // 64)
            assert ((c["th"] - 1) * s + 3) * ((c["tw"] - 1) * s + 3) <= 400 and c["lds"] <= 160 * 1024
            assert c["out"]["c"] == c["K"] and c["out"]["h"] == c["OH"]
        # only the first depthwise convolution (its producer is the 3x3 first layer) runs as a chain of its own
        assert sum(c["kind"] == "dwconv" for c in l3["chains"]) == 1
        # (the byte counts include the partial sums of the reduction splits of the tail, the same at both levels)
        assert l3["hbm_bytes"] < 0.70 * l2["hbm_bytes"]
    assert all(c.get("loader") != "pwdw" for c in l2["chains"])


def test_pattern_depthwise_to_pointwise_on_chip():
    # a depthwise convolution whose pointwise consumer ends the cascade keeps the older link: its result is the
    # operand panel of the pointwise GEMM (ShuffleNet units of the first two stages; the third, 352 channels, is too
    # wide for that kernel and links pointwise -> depthwise instead)
    g = wg.build(5, 1, draw=False)
    l3 = plan_json(g, link=3, compute=X.XENOS_BF16)["plan"]
    dwpw = [c for c in l3["chains"] if c.get("dw_linked") and c.get("loader") == "vector"]
    pwdw = [c for c in l3["chains"] if c.get("loader") == "pwdw"]
    assert len(dwpw) >= 12 and len(pwdw) == 4
    for c in dwpw:
        k = _kinds(g, c)
        assert k[0] == "conv" and g.ops[c["ops"][0]].attrs["groups"] > 1 and k.count("conv") == 2
    for c in pwdw:
        assert c["K"] == 352 and _kinds(g, c).count("conv") == 2


def test_pattern_first_layer_pair_on_chip():
    g = wg.build(3, 2, draw=False)
    l3 = plan_json(g, link=3, compute=X.XENOS_BF16)["plan"]
    c0 = l3["chains"][0]
    assert c0["loader"] == "pair" and _kinds(g, c0) == ["conv", "relu", "conv", "relu", "maxpool"] and c0["in"]["mem"] == "input"
    assert plan_json(g, link=3, compute=X.XENOS_F32)["plan"]["chains"][0]["loader"] == "stem"   # the pair kernel is bf16 only


def test_plan_metadata_names_the_graph_tensor_of_every_view():
    # per-chain checks rely on it: every chain's input / output view says which graph tensor (and channel range) it holds
    for cfg in (1, 2, 4, 5):
        g = wg.build(cfg, 1, draw=False)
        shapes = g.shapes()
        for link in (0, 2, 3):
            q = plan_json(g, link=link, compute=X.XENOS_BF16)["plan"]
            for c in q["chains"]:
                for key in ("in", "in2", "out"):
                    v = c.get(key)
                    if v is None or v["tensor"] < 0:
                        continue
                    n, ch, h, w = shapes[v["tensor"]]
                    assert (v["n"], v["h"], v["w"]) == (n, h, w) and v["c0"] + (v["c"] - 1) * v["cs"] < ch, (cfg, link, c["name"], key, v)
            assert q["chains"][-1]["out"]["tensor"] == g.output and q["chains"][-1]["out"]["mem"] == "output"


def test_pattern_matmul_to_matmul_layout_link():
    # Table 1, MatmulX -> MatmulY: the first matmul's chain (+ ReLU) writes the row-major [row][column] tensor the
    # second one reads as its operand, with no pass in between; bias, ReLU and the shortcut add are operators of the
    # matmul chains, not passes of their own
    g = wg.matmul_chain(rows=128, widths=(512, 2048, 512), draw=False)
    for compute in (X.XENOS_BF16, X.XENOS_F32):
        q = plan_json(g, link=2, compute=compute)["plan"]
        mm = [c for c in q["chains"] if c["kind"] == "conv"]
        assert len(mm) == 2 and _kinds(g, mm[0]) == ["matmul", "relu"] and _kinds(g, mm[1]) == ["matmul", "add"]
        assert mm[0]["N"] == 128 and mm[0]["K"] == 2048 and mm[1]["C"] == 2048 and mm[1]["K"] == 512
        # (where the first matmul shares its reduction out over workgroups, its summing pass is the launch that finishes the
        # chain and writes the tensor)
        between = [c for c in q["chains"] if mm[0]["i"] < c["i"] < mm[1]["i"]]
        assert [c["kind"] for c in between] in ([], ["splitk_finish"]) and all(c["ops"] == mm[0]["ops"] for c in between)
        o, i = (between[0] if between else mm[0])["out"], mm[1]["in"]
        assert o["mem"] == i["mem"] == "workspace" and o["byte_off"] == i["byte_off"] and (o["sN"], o["sP"], o["sK"]) == (2048, 2048, 1) == (i["sN"], i["sP"], i["sK"])
        u0 = plan_json(g, link=0, compute=compute)["plan"]
        assert u0["n_chains"] > q["n_chains"] and u0["hbm_bytes"] > q["hbm_bytes"]
    # shape errors of the operator
    keep = []
    bad = wg.matmul_chain(rows=4, widths=(8, 8), residual=False, draw=False)
    ops = X.op_descs(bad, keep)
    with pytest.raises(X.XenosError) as e:
        X.xenos_graph_create(X.TensorDesc(4, 2, 2, 2, X.XENOS_F32, X.XENOS_NCHW), ops, 1)     # not a rows x columns tensor
    assert e.value.status == X.XENOS_ESHAPE
