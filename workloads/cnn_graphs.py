"""Seeded synthetic CNN compute graphs (shapes and value distributions only).

This module is the one thing the fp64 CPU oracle and the HIP path share: it
describes a CNN as a topologically ordered list of operator records with
seeded fp32 parameters, in the vocabulary of the paper's operator library
(Table 3: conv, bn/bias/relu which fuse to CBR, max/avg/global pooling, add,
concat, matmul/FC).  It contains none of the method's arithmetic: no
convolution, folding, linking or tiling happens here.

Tensor ids: 0 is the graph input, i + 1 is the output of ops[i].

The five workloads stand in for the model families the paper evaluates
(Section 7.1: MobileNet, ResNet18, SqueezeNet, ...) with the public
architectures' shapes and random values; no trained weights or dataset images
are involved (inference time does not depend on values).

Value recipe (He-normal = N(0, std = sqrt(2 / fan_in)), fan_in = C/groups*R*S):
  input  ~ U[-1, 1];  conv / fc weight ~ He-normal;  bias = 0 unless asked;
  BN: gamma ~ U[0.5, 1.5], beta ~ N(0, 0.1), mean ~ N(0, 0.1), var ~ U[0.5, 1.5],
  eps = 1e-5.
Draw order from one numpy PCG64 stream: input, then per operator in
topological order: weight, bias (only if non-zero biases are requested),
gamma, beta, mean, var.  Seed = 230200282 + 1000 * config + batch.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 230200282


def seed_for(config: int, batch: int) -> int:
    return BASE_SEED + 1000 * int(config) + int(batch)


@dataclass
class Op:
    kind: str                      # conv bias bn relu maxpool avgpool gap add concat fc slice shuffle matmul
    inputs: List[int]
    attrs: Dict[str, float] = field(default_factory=dict)
    params: Dict[str, np.ndarray] = field(default_factory=dict)
    name: str = ""


@dataclass
class Graph:
    name: str
    input_shape: Tuple[int, int, int, int]        # N, C, H, W
    ops: List[Op]
    output: int                                   # tensor id of the graph output
    x: Optional[np.ndarray] = None                # seeded input, fp32 NCHW

    def shapes(self) -> List[Tuple[int, int, int, int]]:
        """Shape (N, C, H, W) of every tensor id; pure integer bookkeeping."""
        out = [tuple(self.input_shape)]
        for op in self.ops:
            out.append(_infer(op, [out[i] for i in op.inputs]))
        return out


def _pool_out(n: int, k: int, s: int, p: int, ceil_mode: int) -> int:
    if ceil_mode:
        o = -(-(n + 2 * p - k) // s) + 1
        if (o - 1) * s >= n + p:      # last window must start inside the input or left padding
            o -= 1
        return o
    return (n + 2 * p - k) // s + 1


def _infer(op: Op, ins):
    a = op.attrs
    n, c, h, w = ins[0]
    if op.kind == "conv":
        oh = (h + 2 * a["pad"] - a["kh"]) // a["stride"] + 1
        ow = (w + 2 * a["pad"] - a["kw"]) // a["stride"] + 1
        return (n, a["out_c"], oh, ow)
    if op.kind in ("bias", "bn", "relu"):
        return (n, c, h, w)
    if op.kind in ("maxpool", "avgpool"):
        return (n, c, _pool_out(h, a["k"], a["stride"], a["pad"], a.get("ceil", 0)),
                _pool_out(w, a["k"], a["stride"], a["pad"], a.get("ceil", 0)))
    if op.kind == "gap":
        return (n, c, 1, 1)
    if op.kind == "add":
        assert ins[0] == ins[1], (ins, op.name)
        return ins[0]
    if op.kind == "concat":
        assert all(i[0] == n and i[2:] == (h, w) for i in ins)
        return (n, sum(i[1] for i in ins), h, w)
    if op.kind == "fc":
        return (n, a["out_c"], 1, 1)
    if op.kind == "matmul":
        assert (h, w) == (1, 1), (ins, op.name)
        return (n, a["out_c"], 1, 1)
    if op.kind == "slice":
        assert 0 <= a["c_begin"] and a["out_c"] >= 1 and a["c_begin"] + a["out_c"] <= c, (ins, a)
        return (n, a["out_c"], h, w)
    if op.kind == "shuffle":
        assert a["groups"] >= 1 and c % a["groups"] == 0, (ins, a)
        return (n, c, h, w)
    raise ValueError(op.kind)


class _Builder:
    """Appends operators and draws their parameters in the documented order."""

    def __init__(self, name, input_shape, seed, nonzero_bias=False, draw=True):
        self.rng = np.random.default_rng(seed)
        self.g = Graph(name, tuple(input_shape), [], 0)
        self.draw = draw
        self.nonzero_bias = nonzero_bias
        self.g.x = self._uniform(input_shape, -1.0, 1.0)
        self._shapes = [tuple(input_shape)]

    # -- random draws (all fp32) ------------------------------------------
    def _normal(self, shape, std):
        if not self.draw:
            return np.zeros(shape, np.float32)
        return (self.rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)

    def _uniform(self, shape, lo, hi):
        if not self.draw:
            return np.zeros(shape, np.float32)
        return (self.rng.random(shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)).astype(np.float32)

    # -- operators ----------------------------------------------------------
    def _push(self, op: Op) -> int:
        self.g.ops.append(op)
        self._shapes.append(_infer(op, [self._shapes[i] for i in op.inputs]))
        return len(self.g.ops)

    def shape(self, t):
        return self._shapes[t]

    def conv(self, x, out_c, k, stride=1, pad=0, groups=1, name="", bias=None):
        c = self._shapes[x][1]
        fan_in = (c // groups) * k * k
        p = {"weight": self._normal((out_c, c // groups, k, k), math.sqrt(2.0 / fan_in))}
        want_bias = self.nonzero_bias if bias is None else bias
        if want_bias:
            p["bias"] = self._normal((out_c,), 0.1)
        return self._push(Op("conv", [x], dict(out_c=out_c, kh=k, kw=k, stride=stride, pad=pad,
                                                groups=groups), p, name))

    def bias(self, x, name=""):
        c = self._shapes[x][1]
        return self._push(Op("bias", [x], {}, {"bias": self._normal((c,), 0.1)}, name))

    def bn(self, x, name=""):
        c = self._shapes[x][1]
        p = {"gamma": self._uniform((c,), 0.5, 1.5), "beta": self._normal((c,), 0.1),
             "mean": self._normal((c,), 0.1), "var": self._uniform((c,), 0.5, 1.5)}
        return self._push(Op("bn", [x], {"eps": 1e-5}, p, name))

    def relu(self, x, name=""):
        return self._push(Op("relu", [x], {}, {}, name))

    def maxpool(self, x, k, stride, pad=0, ceil=0, name=""):
        return self._push(Op("maxpool", [x], dict(k=k, stride=stride, pad=pad, ceil=ceil), {}, name))

    def avgpool(self, x, k, stride, pad=0, ceil=0, count_include_pad=0, name=""):
        return self._push(Op("avgpool", [x], dict(k=k, stride=stride, pad=pad, ceil=ceil,
                                                   count_include_pad=count_include_pad), {}, name))

    def gap(self, x, name=""):
        return self._push(Op("gap", [x], {}, {}, name))

    def add(self, a, b, name=""):
        return self._push(Op("add", [a, b], {}, {}, name))

    def concat(self, xs, name=""):
        return self._push(Op("concat", list(xs), {}, {}, name))

    def slice(self, x, c_begin, out_c, name=""):
        """Channels [c_begin, c_begin + out_c) of x."""
        return self._push(Op("slice", [x], dict(c_begin=c_begin, out_c=out_c), {}, name))

    def shuffle(self, x, groups, name=""):
        """Channel shuffle: the channels seen as [groups][C / groups] are written out as [C / groups][groups]."""
        return self._push(Op("shuffle", [x], dict(groups=groups), {}, name))

    def fc(self, x, out_c, name="", bias=None):
        n, c, h, w = self._shapes[x]
        fan_in = c * h * w
        p = {"weight": self._normal((out_c, fan_in), math.sqrt(2.0 / fan_in))}
        want_bias = self.nonzero_bias if bias is None else bias
        if want_bias:
            p["bias"] = self._normal((out_c,), 0.1)
        return self._push(Op("fc", [x], dict(out_c=out_c), p, name))

    def matmul(self, x, out_c, name="", bias=None):
        """Y[M][out_c] = X[M][K] . W[out_c][K]^T (+ bias) on an M x K x 1 x 1 tensor (rows x columns)."""
        m, k, h, w = self._shapes[x]
        assert (h, w) == (1, 1)
        p = {"weight": self._normal((out_c, k), math.sqrt(2.0 / k))}
        want_bias = self.nonzero_bias if bias is None else bias
        if want_bias:
            p["bias"] = self._normal((out_c,), 0.1)
        return self._push(Op("matmul", [x], dict(out_c=out_c), p, name))

    def cbr(self, x, out_c, k, stride=1, pad=0, groups=1, name="", bn=True, relu=True):
        t = self.conv(x, out_c, k, stride, pad, groups, name)
        if bn:
            t = self.bn(t, name + ".bn")
        if relu:
            t = self.relu(t, name + ".relu")
        return t

    def finish(self, out) -> Graph:
        self.g.output = out
        return self.g


# ---------------------------------------------------------------------------
# The five workloads
# ---------------------------------------------------------------------------

def single_chain(batch=1, seed=None, hw=32, in_c=3, out_c=16, nonzero_bias=False, draw=True) -> Graph:
    """Config 0: Conv3x3 s1 p1 -> BN -> ReLU -> MaxPool2x2 s2 (the paper's CBRM, Table 3)."""
    b = _Builder("single_chain", (batch, in_c, hw, hw), seed_for(0, batch) if seed is None else seed,
                 nonzero_bias, draw)
    t = b.cbr(0, out_c, 3, 1, 1, name="c0")
    t = b.maxpool(t, 2, 2, name="pool")
    return b.finish(t)


MOBILENET_BLOCKS = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2),
                    (512, 1), (512, 1), (512, 1), (512, 1), (512, 1), (1024, 2), (1024, 1)]


def mobilenet_v1(batch=1, seed=None, hw=224, width=1.0, classes=1000, nonzero_bias=False, draw=True) -> Graph:
    """Config 1: depthwise-separable stack (the paper's Section 2.2 / Figure 5 example family)."""
    b = _Builder("mobilenet_v1", (batch, 3, hw, hw), seed_for(1, batch) if seed is None else seed,
                 nonzero_bias, draw)
    ch = lambda c: max(8, int(c * width))
    t = b.cbr(0, ch(32), 3, 2, 1, name="conv0")
    for i, (oc, s) in enumerate(MOBILENET_BLOCKS, 1):
        c = b.shape(t)[1]
        t = b.cbr(t, c, 3, s, 1, groups=c, name=f"dw{i}")
        t = b.cbr(t, ch(oc), 1, 1, 0, name=f"pw{i}")
    t = b.gap(t, "gap")
    t = b.fc(t, classes, "fc")
    return b.finish(t)


def resnet18(batch=1, seed=None, hw=224, width=1.0, classes=1000, nonzero_bias=False, draw=True) -> Graph:
    """Config 2: BasicBlock backbone; exercises the shortcut-connection linking pattern (Table 1)."""
    b = _Builder("resnet18", (batch, 3, hw, hw), seed_for(2, batch) if seed is None else seed,
                 nonzero_bias, draw)
    ch = lambda c: max(8, int(c * width))
    t = b.cbr(0, ch(64), 7, 2, 3, name="conv1")
    t = b.maxpool(t, 3, 2, 1, name="pool1")
    for si, c in enumerate((64, 128, 256, 512), 1):
        for bi in range(2):
            stride = 2 if (si > 1 and bi == 0) else 1
            name = f"s{si}b{bi}"
            skip = t
            u = b.cbr(t, ch(c), 3, stride, 1, name=name + ".c1")
            u = b.cbr(u, ch(c), 3, 1, 1, name=name + ".c2", relu=False)
            if stride != 1 or b.shape(skip)[1] != ch(c):
                skip = b.cbr(skip, ch(c), 1, stride, 0, name=name + ".proj", relu=False)
            u = b.add(u, skip, name + ".add")
            t = b.relu(u, name + ".out")
    t = b.gap(t, "gap")
    t = b.fc(t, classes, "fc")
    return b.finish(t)


VGG_GROUPS = [(64, 2), (128, 2), (256, 3), (512, 3), (512, 3)]


def vgg16(batch=32, seed=None, hw=224, width=1.0, fc_dim=4096, classes=1000, nonzero_bias=False,
          draw=True) -> Graph:
    """Config 3: plain Conv3x3+ReLU stack, MaxPool2x2 ending each group, three FC layers."""
    b = _Builder("vgg16", (batch, 3, hw, hw), seed_for(3, batch) if seed is None else seed,
                 nonzero_bias, draw)
    ch = lambda c: max(8, int(c * width))
    t = 0
    for gi, (c, n) in enumerate(VGG_GROUPS, 1):
        for ci in range(1, n + 1):
            t = b.cbr(t, ch(c), 3, 1, 1, name=f"g{gi}c{ci}", bn=False)
        t = b.maxpool(t, 2, 2, name=f"pool{gi}")
    t = b.fc(t, fc_dim, "fc6")
    t = b.relu(t, "fc6.relu")
    t = b.fc(t, fc_dim, "fc7")
    t = b.relu(t, "fc7.relu")
    t = b.fc(t, classes, "fc8")
    return b.finish(t)


SQUEEZE = [16, 16, 32, 32, 48, 48, 64, 64]


def squeezenet11(batch=1, seed=None, hw=224, classes=1000, nonzero_bias=False, draw=True) -> Graph:
    """Config 4: Fire modules; exercises linking across concat and fan-out of a shared producer."""
    b = _Builder("squeezenet11", (batch, 3, hw, hw), seed_for(4, batch) if seed is None else seed,
                 nonzero_bias, draw)
    t = b.cbr(0, 64, 3, 2, 0, name="conv1", bn=False)
    t = b.maxpool(t, 3, 2, 0, ceil=1, name="pool1")
    for i, s in enumerate(SQUEEZE, 1):
        q = b.cbr(t, s, 1, name=f"f{i}.sq", bn=False)
        e1 = b.cbr(q, 4 * s, 1, name=f"f{i}.e1", bn=False)
        e3 = b.cbr(q, 4 * s, 3, 1, 1, name=f"f{i}.e3", bn=False)
        t = b.concat([e1, e3], f"f{i}.cat")
        if i in (2, 4):
            t = b.maxpool(t, 3, 2, 0, ceil=1, name=f"pool_f{i}")
    t = b.cbr(t, classes, 1, name="conv10", bn=False)
    t = b.gap(t, "gap")
    return b.finish(t)


def shufflenet_v2(batch=1, seed=None, hw=224, channels=(176, 352, 704), repeats=(4, 8, 4), stem=24, last=1024,
                  classes=1000, nonzero_bias=False, draw=True) -> Graph:
    """ShuffleNet-style graph (one of the paper's seven evaluation models, Section 7.1): units that split the channels in
    two halves, run a 1x1 -> depthwise 3x3 -> 1x1 branch on one half, concatenate and shuffle the channels in two groups.
    The shuffle moves no data when linked: it is the order in which the two halves are written."""
    b = _Builder("shufflenet_v2", (batch, 3, hw, hw), seed_for(5, batch) if seed is None else seed, nonzero_bias, draw)
    t = b.cbr(0, stem, 3, 2, 1, name="conv1")
    t = b.maxpool(t, 3, 2, 1, name="pool1")
    for si, (c, reps) in enumerate(zip(channels, repeats), 2):
        h = c // 2
        for u in range(reps):
            nm = f"s{si}u{u}"
            if u == 0:           # down-sampling unit: both branches read the whole input
                l = b.cbr(t, b.shape(t)[1], 3, 2, 1, groups=b.shape(t)[1], name=nm + ".l.dw", relu=False)
                l = b.cbr(l, h, 1, name=nm + ".l.pw")
                r = b.cbr(t, h, 1, name=nm + ".r.pw1")
                r = b.cbr(r, h, 3, 2, 1, groups=h, name=nm + ".r.dw", relu=False)
                r = b.cbr(r, h, 1, name=nm + ".r.pw2")
            else:
                l = b.slice(t, 0, h, nm + ".lo")
                r = b.slice(t, h, h, nm + ".hi")
                r = b.cbr(r, h, 1, name=nm + ".r.pw1")
                r = b.cbr(r, h, 3, 1, 1, groups=h, name=nm + ".r.dw", relu=False)
                r = b.cbr(r, h, 1, name=nm + ".r.pw2")
            t = b.shuffle(b.concat([l, r], nm + ".cat"), 2, nm + ".shuffle")
    t = b.cbr(t, last, 1, name="conv5")
    t = b.gap(t, "gap")
    t = b.fc(t, classes, "fc")
    return b.finish(t)


# Operator micro-benchmark shapes (Table 4): name -> (feature map H, W, C; kernel R, S; out channels K; what follows)
TABLE4 = {
    "cbr_maxpool": (224, 224, 3, 3, 3, 24, "maxpool"),      # printed with inC 24 / outC 224; read as 3 -> 24 (inC must be 3)
    "cbr_avgpool": (7, 7, 1024, 1, 1, 1024, "gap"),         # CBRA: pointwise conv + global average (MobileNet tail)
    "fully_connected": (1, 1, 1536, 1, 1, 1000, "fc"),
    "cbr": (112, 112, 32, 1, 1, 64, "none"),
}


def table4(name: str, batch=1, seed=None, nonzero_bias=False, draw=True) -> Graph:
    """One operator of the paper's micro-benchmark (Table 4) as a graph of its own."""
    h, w, c, r, s_, k, tail = TABLE4[name]
    idx = sorted(TABLE4).index(name)
    b = _Builder("table4_" + name, (batch, c, h, w), seed_for(10 + idx, batch) if seed is None else seed, nonzero_bias, draw)
    if tail == "fc":
        t = b.fc(0, k, name="fc")
    else:
        t = b.cbr(0, k, r, 1, r // 2, name="c0")
        if tail == "maxpool":
            t = b.maxpool(t, 2, 2, name="pool")
        elif tail == "gap":
            t = b.gap(t, name="gap")
    return b.finish(t)


def matmul_chain(rows=128, widths=(512, 2048, 512), seed=None, residual=True, nonzero_bias=True, draw=True) -> Graph:
    """MatmulX -> MatmulY chains (Table 1, last row; the transformer / LSTM workloads of Section 7.1 are made of them): the
    feed-forward block of a small BERT is rows x 512 -> 2048 -> 512 with a ReLU in between and a shortcut around it.
    widths = (K, N1, N2, ...): one matmul per step, ReLU between them.  With residual (and equal first and last width) a
    BN + ReLU pre-activation comes first and is added to the last result, as the block's shortcut."""
    b = _Builder("matmul_chain", (rows, widths[0], 1, 1), seed_for(20, rows) if seed is None else seed, nonzero_bias, draw)
    shortcut = residual and widths[-1] == widths[0]
    x0 = b.relu(b.bn(0, "pre.bn"), "pre.relu") if shortcut else 0
    t = x0
    for i, n_out in enumerate(widths[1:], 1):
        t = b.matmul(t, n_out, name=f"mm{i}")
        if i < len(widths) - 1:
            t = b.relu(t, f"mm{i}.relu")
    if shortcut:
        t = b.add(t, x0, "shortcut")
    return b.finish(t)


CONFIGS = {0: single_chain, 1: mobilenet_v1, 2: resnet18, 3: vgg16, 4: squeezenet11, 5: shufflenet_v2}


def build(config: int, batch: int, **kw) -> Graph:
    return CONFIGS[config](batch=batch, **kw)


# ---------------------------------------------------------------------------
# Shape-only bookkeeping used by the bench report (no arithmetic on values)
# ---------------------------------------------------------------------------

def conv_fc_flops(g: Graph) -> int:
    """2 * MACs of the conv and fc operators (the paper's operators x.conv / x.matmul)."""
    shp = g.shapes()
    total = 0
    for i, op in enumerate(g.ops):
        n, k, oh, ow = shp[i + 1]
        if op.kind == "conv":
            c = shp[op.inputs[0]][1] // op.attrs["groups"]
            total += 2 * n * k * oh * ow * c * op.attrs["kh"] * op.attrs["kw"]
        elif op.kind == "fc":
            _, c, h, w = shp[op.inputs[0]]
            total += 2 * n * k * c * h * w
    return total


def builder(name: str, input_shape, seed: int, nonzero_bias: bool = False) -> _Builder:
    """A builder for ad-hoc graphs (unit chains in the tests); same draw rules as the five workloads."""
    return _Builder(name, input_shape, seed, nonzero_bias)
