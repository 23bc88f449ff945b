"""ctypes front end of the fp64 CPU oracle (oracle/xenos_oracle.c) and a graph runner.

TEST INFRASTRUCTURE ONLY: importable from tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg; the product package never imports it.

run_graph() applies the operators of a workloads.cnn_graphs.Graph one by one, in
graph order, on NCHW float64 arrays: the un-linked, un-split, un-fused model that
the paper's optimised model must be equivalent to (Section 3).  fp32 seeded
parameters are widened to float64 and never rounded to a narrower type.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xenos_oracle.c")
_LIB = os.path.join(_HERE, "libxenos_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.xo_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(lib().xo_threads())


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.cast(None, _D)
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(_D)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def pool_out(n: int, k: int, s: int, p: int, ceil_mode: int) -> int:
    """Output length of a pooling window sweep (floor mode, or ceil mode with the rule that the
    last window must start inside the input or its left padding)."""
    if ceil_mode:
        o = -(-(n + 2 * p - k) // s) + 1
        if (o - 1) * s >= n + p:
            o -= 1
        return o
    return (n + 2 * p - k) // s + 1


def conv2d(x, w, bias=None, stride=1, pad=0, groups=1) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    b = None if bias is None else _f64(bias)
    n, c, h, wd = x.shape
    k, cg, r, s = w.shape
    assert cg * groups == c and k % groups == 0
    oh, ow = (h + 2 * pad - r) // stride + 1, (wd + 2 * pad - s) // stride + 1
    y = np.empty((n, k, oh, ow), np.float64)
    lib().xo_conv2d(_p(x), n, c, h, wd, _p(w), _p(b), k, r, s, stride, stride, pad, pad, groups, _p(y))
    return y


def bias_add(x, b) -> np.ndarray:
    x, b = _f64(x), _f64(b)
    y = np.empty_like(x)
    lib().xo_bias(_p(x), *x.shape, _p(b), _p(y))
    return y


def bn(x, gamma, beta, mean, var, eps=1e-5) -> np.ndarray:
    x = _f64(x)
    y = np.empty_like(x)
    lib().xo_bn(_p(x), *x.shape, _p(_f64(gamma)), _p(_f64(beta)), _p(_f64(mean)), _p(_f64(var)),
                ctypes.c_double(eps), _p(y))
    return y


def relu(x) -> np.ndarray:
    x = _f64(x)
    y = np.empty_like(x)
    lib().xo_relu(_p(x), ctypes.c_size_t(x.size), _p(y))
    return y


def pool(x, k, stride, pad=0, ceil=0, avg=False, count_include_pad=0) -> np.ndarray:
    x = _f64(x)
    n, c, h, w = x.shape
    oh, ow = pool_out(h, k, stride, pad, ceil), pool_out(w, k, stride, pad, ceil)
    y = np.empty((n, c, oh, ow), np.float64)
    lib().xo_pool(_p(x), n, c, h, w, k, k, stride, stride, pad, pad, oh, ow, int(bool(avg)),
                  int(count_include_pad), _p(y))
    return y


def gap(x) -> np.ndarray:
    x = _f64(x)
    n, c, h, w = x.shape
    y = np.empty((n, c, 1, 1), np.float64)
    lib().xo_gap(_p(x), n, c, h, w, _p(y))
    return y


def add(a, b) -> np.ndarray:
    a, b = _f64(a), _f64(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().xo_add(_p(a), _p(b), ctypes.c_size_t(a.size), _p(y))
    return y


def concat(xs) -> np.ndarray:
    xs = [_f64(x) for x in xs]
    n, _, h, w = xs[0].shape
    ct = sum(x.shape[1] for x in xs)
    y = np.empty((n, ct, h, w), np.float64)
    c0 = 0
    for x in xs:
        lib().xo_concat_part(_p(x), n, x.shape[1], h * w, c0, ct, _p(y))
        c0 += x.shape[1]
    return y


def channel_slice(x, c_begin, out_c) -> np.ndarray:
    """Channels [c_begin, c_begin + out_c) of an NCHW tensor (the inverse of concat: Section 4.2.2, Eq. 1 read backwards)."""
    x = _f64(x)
    assert 0 <= c_begin and out_c >= 1 and c_begin + out_c <= x.shape[1]
    y = np.empty((x.shape[0], out_c) + x.shape[2:], np.float64)
    for k in range(out_c):
        y[:, k] = x[:, c_begin + k]
    return y


def channel_shuffle(x, groups) -> np.ndarray:
    """Channel shuffle of the ShuffleNet models (Section 7.1 lists ShuffleNet; the paper gives no formula, this is the
    operator's published definition): with C = groups * m, output channel i * groups + j is input channel j * m + i."""
    x = _f64(x)
    c = x.shape[1]
    assert groups >= 1 and c % groups == 0
    m = c // groups
    y = np.empty_like(x)
    for j in range(groups):
        for i in range(m):
            y[:, i * groups + j] = x[:, j * m + i]
    return y


def fc(x, w, bias=None) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    n = x.shape[0]
    xi = x.reshape(n, -1)                       # NCHW flatten: i = c*H*W + h*W + w
    o, i = w.shape
    assert xi.shape[1] == i
    b = None if bias is None else _f64(bias)
    y = np.empty((n, o), np.float64)
    lib().xo_fc(_p(np.ascontiguousarray(xi)), n, i, _p(w), _p(b), o, _p(y))
    return y.reshape(n, o, 1, 1)


def matmul(x, w, bias=None) -> np.ndarray:
    """x.matmul (Table 3): Y[M][N] = X[M][K] . W[N][K]^T (+ bias[N]) on an M x K x 1 x 1 tensor, whose first dimension
    are the rows: the fully connected definition on a 1x1 map, written out as such."""
    x, w = _f64(x), _f64(w)
    assert x.ndim == 4 and x.shape[2:] == (1, 1), x.shape
    m, k = x.shape[0], x.shape[1]
    n, k2 = w.shape
    assert k == k2
    b = None if bias is None else _f64(bias)
    y = np.empty((m, n), np.float64)
    lib().xo_fc(_p(np.ascontiguousarray(x.reshape(m, k))), m, k, _p(w), _p(b), n, _p(y))
    return y.reshape(m, n, 1, 1)


def apply_op(op, ins: List[np.ndarray]) -> np.ndarray:
    """One operator of the graph, by its plain definition."""
    a, p = op.attrs, op.params
    if op.kind == "conv":
        return conv2d(ins[0], p["weight"], p.get("bias"), a["stride"], a["pad"], a["groups"])
    if op.kind == "bias":
        return bias_add(ins[0], p["bias"])
    if op.kind == "bn":
        return bn(ins[0], p["gamma"], p["beta"], p["mean"], p["var"], a["eps"])
    if op.kind == "relu":
        return relu(ins[0])
    if op.kind == "maxpool":
        return pool(ins[0], a["k"], a["stride"], a["pad"], a.get("ceil", 0), avg=False)
    if op.kind == "avgpool":
        return pool(ins[0], a["k"], a["stride"], a["pad"], a.get("ceil", 0), avg=True,
                    count_include_pad=a.get("count_include_pad", 0))
    if op.kind == "gap":
        return gap(ins[0])
    if op.kind == "add":
        return add(ins[0], ins[1])
    if op.kind == "concat":
        return concat(ins)
    if op.kind == "fc":
        return fc(ins[0], p["weight"], p.get("bias"))
    if op.kind == "matmul":
        return matmul(ins[0], p["weight"], p.get("bias"))
    if op.kind == "slice":
        return channel_slice(ins[0], a["c_begin"], a["out_c"])
    if op.kind == "shuffle":
        return channel_shuffle(ins[0], a["groups"])
    raise ValueError(op.kind)


def run_graph(g, x=None, keep: Optional[List[int]] = None) -> Dict[int, np.ndarray]:
    """Run every operator in graph order. Returns {tensor id: NCHW float64 array} for the graph
    output and every id in `keep` (all tensors if keep == 'all'); other intermediates are freed
    as soon as their last consumer has run."""
    x = g.x if x is None else x
    last_use = {}
    for i, op in enumerate(g.ops):
        for t in op.inputs:
            last_use[t] = i
    keep_all = keep == "all"
    keep_set = set() if keep is None or keep_all else set(keep)
    keep_set.add(g.output)
    live = {0: _f64(x)}
    out = {}
    for i, op in enumerate(g.ops):
        y = apply_op(op, [live[t] for t in op.inputs])
        live[i + 1] = y
        for t in set(op.inputs):
            if last_use[t] == i and not (keep_all or t in keep_set):
                del live[t]
    for t, v in live.items():
        if keep_all or t in keep_set:
            out[t] = v
    return out


def forward(g, x=None) -> np.ndarray:
    return run_graph(g, x)[g.output]
