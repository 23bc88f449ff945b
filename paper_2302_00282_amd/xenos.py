"""Thin ctypes binding of libxenos.so: argument marshalling only.

The functions carry the names of the C ABI (include/xenos.h).  Every step of the hot path runs
in the HIP kernels behind that ABI; PyTorch appears only in `Session`, which owns the device
buffers (weights, workspace, input, output) and supplies the stream.  If the shared library is
missing the import of this module's functions fails loudly -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import json
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxenos.so")

XENOS_OK, XENOS_EINVAL, XENOS_ESHAPE, XENOS_EUNSUPPORTED, XENOS_ENOMEM, XENOS_EDEVICE = range(6)
XENOS_F32, XENOS_BF16 = 0, 1
XENOS_NCHW, XENOS_NHWC = 0, 1
(XENOS_OP_CONV, XENOS_OP_BIAS, XENOS_OP_BN, XENOS_OP_RELU, XENOS_OP_MAXPOOL, XENOS_OP_AVGPOOL,
 XENOS_OP_GLOBAL_AVGPOOL, XENOS_OP_ADD, XENOS_OP_CONCAT, XENOS_OP_FC, XENOS_OP_SLICE, XENOS_OP_SHUFFLE, XENOS_OP_MATMUL) = range(13)

_KIND = {"conv": XENOS_OP_CONV, "bias": XENOS_OP_BIAS, "bn": XENOS_OP_BN, "relu": XENOS_OP_RELU,
         "maxpool": XENOS_OP_MAXPOOL, "avgpool": XENOS_OP_AVGPOOL, "gap": XENOS_OP_GLOBAL_AVGPOOL,
         "add": XENOS_OP_ADD, "concat": XENOS_OP_CONCAT, "fc": XENOS_OP_FC, "slice": XENOS_OP_SLICE,
         "shuffle": XENOS_OP_SHUFFLE, "matmul": XENOS_OP_MATMUL}

_FP = C.POINTER(C.c_float)


class TensorDesc(C.Structure):
    _fields_ = [("n", C.c_int), ("c", C.c_int), ("h", C.c_int), ("w", C.c_int),
                ("dtype", C.c_int), ("layout", C.c_int)]


class OpDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("n_inputs", C.c_int), ("inputs", C.c_int * 4),
                ("out_c", C.c_int), ("kh", C.c_int), ("kw", C.c_int),
                ("stride_h", C.c_int), ("stride_w", C.c_int), ("pad_h", C.c_int), ("pad_w", C.c_int),
                ("groups", C.c_int), ("ceil_mode", C.c_int), ("count_include_pad", C.c_int), ("c_begin", C.c_int),
                ("eps", C.c_float),
                ("weight", _FP), ("bias", _FP), ("gamma", _FP), ("beta", _FP), ("mean", _FP), ("var", _FP)]


class HwInfo(C.Structure):
    _fields_ = [("num_cu", C.c_int), ("lds_bytes_per_cu", C.c_size_t), ("l2_bytes", C.c_size_t),
                ("llc_bytes", C.c_size_t), ("hbm_bytes", C.c_size_t)]


class PlanOpts(C.Structure):
    _fields_ = [("link", C.c_int), ("split", C.c_int), ("compute", C.c_int), ("tile", C.c_int)]


class XenosError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"xenos status {status}: {msg}")
        self.status = status


_lib = None


def lib():
    """Loads libxenos.so; raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_00282_amd.build` "
                              "(hipcc, gfx950); there is no CPU fallback")
        # PyTorch provides the device memory and streams, so the library must share the HIP runtime that
        # torch loads (both have the same soname; the first one loaded serves the whole process).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.xenos_graph_create.argtypes = [C.POINTER(TensorDesc), C.POINTER(OpDesc), C.c_int, C.c_int,
                                         C.POINTER(TensorDesc), C.POINTER(vp)]
        L.xenos_plan_link_split.argtypes = [vp, C.POINTER(HwInfo), C.POINTER(PlanOpts), C.POINTER(vp)]
        L.xenos_plan_query.argtypes = [vp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(TensorDesc),
                                       C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]
        L.xenos_plan_bind.argtypes = [vp, vp, vp, vp]
        L.xenos_run.argtypes = [vp, vp, vp, vp]
        L.xenos_run_graph.argtypes = [vp, vp, vp, vp]
        L.xenos_run_static.argtypes = [vp, vp, vp, vp]
        L.xenos_run_with.argtypes = [vp, vp, vp, vp, vp]
        L.xenos_run_chain.argtypes = [vp, C.c_int, vp, vp, vp]
        L.xenos_plan_tune.argtypes = [vp, vp, vp, vp, C.c_int, C.POINTER(C.c_int)]
        L.xenos_probe_mfma.argtypes = [C.POINTER(HwInfo), vp, C.c_size_t, C.c_int, C.c_int, vp, C.POINTER(C.c_double)]
        L.xenos_probe_read.argtypes = [C.POINTER(HwInfo), vp, C.c_size_t, vp, C.c_size_t, vp]
        L.xenos_destroy.argtypes = [vp]
        L.xenos_destroy.restype = None
        L.xenos_last_error.restype = C.c_char_p
        for f in ("xenos_graph_create", "xenos_plan_link_split", "xenos_plan_query", "xenos_plan_bind",
                  "xenos_run", "xenos_run_graph", "xenos_run_static", "xenos_run_with", "xenos_run_chain", "xenos_plan_tune",
                  "xenos_probe_mfma", "xenos_probe_read"):
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def xenos_last_error() -> str:
    return lib().xenos_last_error().decode()


def _check(st: int):
    if st != XENOS_OK:
        raise XenosError(st, xenos_last_error())


# MI355X: 256 CUs, 160 KiB LDS per CU, 4 MiB L2 per XCD, 256 MiB Infinity Cache, 288 GB HBM3E
MI355X = dict(num_cu=256, lds_bytes_per_cu=160 * 1024, l2_bytes=4 << 20, llc_bytes=256 << 20, hbm_bytes=288 * 10**9)


def xenos_graph_create(input_desc: TensorDesc, ops: Sequence[OpDesc], output_tensor_id: int,
                       output_desc: Optional[TensorDesc] = None) -> int:
    arr = (OpDesc * len(ops))(*ops)
    h = C.c_void_p()
    _check(lib().xenos_graph_create(C.byref(input_desc), arr, len(ops), output_tensor_id,
                                    C.byref(output_desc) if output_desc is not None else None, C.byref(h)))
    return h.value


def xenos_plan_link_split(graph: int, hw: Optional[dict] = None, link: int = 2, split: int = 1,
                          compute: int = XENOS_F32, tile: int = 0) -> int:
    hwi = HwInfo(**(hw or MI355X))
    opts = PlanOpts(link, split, compute, tile)
    h = C.c_void_p()
    _check(lib().xenos_plan_link_split(graph, C.byref(hwi), C.byref(opts), C.byref(h)))
    return h.value


def xenos_plan_query(plan: int) -> dict:
    wb, ws, n = C.c_size_t(), C.c_size_t(), C.c_size_t()
    od = TensorDesc()
    _check(lib().xenos_plan_query(plan, C.byref(wb), C.byref(ws), C.byref(od), None, 0, C.byref(n)))
    buf = C.create_string_buffer(n.value)
    _check(lib().xenos_plan_query(plan, None, None, None, buf, n.value, None))
    return dict(weight_bytes=wb.value, workspace_bytes=ws.value,
                out_desc=dict(n=od.n, c=od.c, h=od.h, w=od.w, dtype=od.dtype, layout=od.layout),
                plan=json.loads(buf.value.decode()))


def xenos_plan_bind(plan: int, d_weights: int, d_workspace: int, stream: int = 0):
    _check(lib().xenos_plan_bind(plan, d_weights, d_workspace, stream))


def xenos_run(plan: int, d_input: int, d_output: int, stream: int = 0):
    _check(lib().xenos_run(plan, d_input, d_output, stream))


def xenos_run_graph(plan: int, d_input: int, d_output: int, stream: int = 0):
    _check(lib().xenos_run_graph(plan, d_input, d_output, stream))


XENOS_STATIC_WORKSPACE_BYTES = 32 << 20


def xenos_run_static(plan: int, d_input: int, d_output: int, stream: int = 0):
    _check(lib().xenos_run_static(plan, d_input, d_output, stream))


def xenos_run_with(plan: int, d_input: int, d_output: int, d_workspace: int, stream: int = 0):
    _check(lib().xenos_run_with(plan, d_input, d_output, d_workspace, stream))


def xenos_plan_tune(plan: int, d_input: int, d_output: int, stream: int = 0, reps: int = 5) -> int:
    """Profiles every legal partition of every tunable chain and keeps the fastest; returns how many choices changed."""
    n = C.c_int(0)
    _check(lib().xenos_plan_tune(plan, d_input, d_output, stream, reps, C.byref(n)))
    return n.value


def xenos_run_chain(plan: int, chain: int, d_input: int, d_output: int, stream: int = 0):
    _check(lib().xenos_run_chain(plan, chain, d_input, d_output, stream))


def xenos_probe_mfma(d_out: int, out_bytes: int, iters: int, stream: int = 0, hw: Optional[dict] = None, data: int = 0) -> float:
    """Enqueues the MFMA-only loop (data: 0 small structured operands, 1 random dense, 2 random with half of the pixel
    operand zero); returns the floating-point operations of the launch."""
    hwi = HwInfo(**(hw or MI355X))
    f = C.c_double(0.0)
    _check(lib().xenos_probe_mfma(C.byref(hwi), d_out, out_bytes, iters, data, stream, C.byref(f)))
    return f.value


def xenos_probe_read(d_in: int, nbytes: int, d_out: int, out_bytes: int, stream: int = 0, hw: Optional[dict] = None):
    hwi = HwInfo(**(hw or MI355X))
    _check(lib().xenos_probe_read(C.byref(hwi), d_in, nbytes, d_out, out_bytes, stream))


def xenos_destroy(handle: Optional[int]):
    if handle:
        lib().xenos_destroy(handle)


# ---------------------------------------------------------------------------------------------
# Marshalling of a workloads.cnn_graphs.Graph (plain records + fp32 numpy arrays) into descriptors
# ---------------------------------------------------------------------------------------------
def _fp(a: Optional[np.ndarray], keep: List[np.ndarray]):
    if a is None:
        return C.cast(None, _FP)
    a = np.ascontiguousarray(a, dtype=np.float32)
    keep.append(a)
    return a.ctypes.data_as(_FP)


def op_descs(g, keep: List[np.ndarray]) -> List[OpDesc]:
    descs = []
    for op in g.ops:
        a, p = op.attrs, op.params
        d = OpDesc()
        d.kind = _KIND[op.kind]
        d.n_inputs = len(op.inputs)
        for j, t in enumerate(op.inputs):
            d.inputs[j] = t
        d.groups = 1
        if op.kind == "conv":
            d.out_c, d.kh, d.kw = a["out_c"], a["kh"], a["kw"]
            d.stride_h = d.stride_w = a["stride"]
            d.pad_h = d.pad_w = a["pad"]
            d.groups = a["groups"]
        elif op.kind in ("maxpool", "avgpool"):
            d.kh = d.kw = a["k"]
            d.stride_h = d.stride_w = a["stride"]
            d.pad_h = d.pad_w = a["pad"]
            d.ceil_mode = a.get("ceil", 0)
            d.count_include_pad = a.get("count_include_pad", 0)
        elif op.kind in ("fc", "matmul"):
            d.out_c = a["out_c"]
        elif op.kind == "slice":
            d.out_c, d.c_begin = a["out_c"], a["c_begin"]
        elif op.kind == "shuffle":
            d.groups = a["groups"]
        elif op.kind == "bn":
            d.eps = a["eps"]
        d.weight = _fp(p.get("weight"), keep)
        d.bias = _fp(p.get("bias"), keep)
        d.gamma = _fp(p.get("gamma"), keep)
        d.beta = _fp(p.get("beta"), keep)
        d.mean = _fp(p.get("mean"), keep)
        d.var = _fp(p.get("var"), keep)
        descs.append(d)
    return descs


def graph_from_workload(g, in_dtype=XENOS_F32, in_layout=XENOS_NCHW, out_dtype=XENOS_F32, out_layout=XENOS_NCHW) -> int:
    keep: List[np.ndarray] = []
    n, c, h, w = g.input_shape
    return xenos_graph_create(TensorDesc(n, c, h, w, in_dtype, in_layout), op_descs(g, keep), g.output,
                              TensorDesc(0, 0, 0, 0, out_dtype, out_layout))


class Session:
    """Owns the device memory of one bound plan (PyTorch tensors) and runs it on torch's current stream.

    in_dtype / in_layout / out_dtype / out_layout are the caller-side formats of the graph input and output
    (XENOS_F32 / XENOS_BF16, XENOS_NCHW / XENOS_NHWC).  set_input() and output() always speak fp32 NCHW numpy: the
    conversion to and from the caller-side format is a torch permute / cast on the device buffers, i.e. what a
    caller holding such tensors would pass; the library reads and writes them in place.
    workspace=False binds no workspace: such a session runs through run_static() only."""

    def __init__(self, g, link=2, split=1, compute=XENOS_F32, tile=0, hw=None, device="cuda:0",
                 in_dtype=XENOS_F32, in_layout=XENOS_NCHW, out_dtype=XENOS_F32, out_layout=XENOS_NCHW, workspace=True):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.in_fmt, self.out_fmt = (in_dtype, in_layout), (out_dtype, out_layout)
        self.graph = graph_from_workload(g, in_dtype, in_layout, out_dtype, out_layout)
        self.plan = None
        try:
            self.plan = xenos_plan_link_split(self.graph, hw, link, split, compute, tile)
            q = xenos_plan_query(self.plan)
            self.info = q["plan"]
            self.out_desc = q["out_desc"]
            self.weights = torch.empty(q["weight_bytes"] + 256, dtype=torch.uint8, device=self.device)
            self.workspace = torch.zeros(q["workspace_bytes"] + 256, dtype=torch.uint8, device=self.device) if workspace else None
            od = self.out_desc
            self.y = self._alloc((od["n"], od["c"], od["h"], od["w"]), out_dtype, out_layout)
            self.x = self._alloc(tuple(g.input_shape), in_dtype, in_layout)
            xenos_plan_bind(self.plan, self._al(self.weights), self._al(self.workspace) if workspace else 0, self.stream())
        except Exception:
            self.close()
            raise

    def _alloc(self, nchw, dtype, layout):
        """A zeroed device tensor of logical shape `nchw`, stored in the given dtype and layout."""
        torch = self.torch
        n, c, h, w = nchw
        shape = (n, h, w, c) if layout == XENOS_NHWC else (n, c, h, w)
        return torch.zeros(shape, dtype=torch.bfloat16 if dtype == XENOS_BF16 else torch.float32, device=self.device)

    @staticmethod
    def _al(t) -> int:
        return (t.data_ptr() + 255) // 256 * 256

    def workspace_view(self):
        """The bound workspace as a uint8 tensor starting at the bound (256-byte aligned) address."""
        off = self._al(self.workspace) - self.workspace.data_ptr()
        return self.workspace[off:]

    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def set_input(self, x: np.ndarray):
        t = self.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
        if self.in_fmt[1] == XENOS_NHWC:
            t = t.permute(0, 2, 3, 1)
        self.x.copy_(t)                      # (the cast to bf16, where asked for, rounds to nearest even)

    def _y_numpy(self) -> np.ndarray:
        y = self.y.float()
        if self.out_fmt[1] == XENOS_NHWC:
            y = y.permute(0, 3, 1, 2)
        return y.contiguous().cpu().numpy()

    def run_static(self):
        xenos_run_static(self.plan, self.x.data_ptr(), self.y.data_ptr(), self.stream())

    def run(self):
        xenos_run(self.plan, self.x.data_ptr(), self.y.data_ptr(), self.stream())

    def run_graph(self):
        xenos_run_graph(self.plan, self.x.data_ptr(), self.y.data_ptr(), self.stream())

    def lane(self) -> "Lane":
        """Device buffers for one more pass of this session's plan in flight (xenos_run_with)."""
        return Lane(self)

    def run_chain(self, i: int):
        xenos_run_chain(self.plan, i, self.x.data_ptr(), self.y.data_ptr(), self.stream())

    def forward(self, x: np.ndarray) -> np.ndarray:
        self.set_input(x)
        self.run()
        self.torch.cuda.synchronize(self.device)
        return self._y_numpy()

    def tune(self, reps: int = 5) -> int:
        """xenos_plan_tune on the session's current input; refreshes `info`."""
        n = xenos_plan_tune(self.plan, self.x.data_ptr(), self.y.data_ptr(), self.stream(), reps)
        self.info = xenos_plan_query(self.plan)["plan"]
        return n

    def output(self) -> np.ndarray:
        """Synchronises and returns the output buffer of the last run / run_graph."""
        self.torch.cuda.synchronize(self.device)
        return self._y_numpy()

    def close(self):
        xenos_destroy(self.plan)
        xenos_destroy(self.graph)
        self.plan = self.graph = None


class Lane:
    """An input, an output and a workspace of their own for passes of a Session's plan that run beside the session's
    passes (xenos_run_with): the weights are the session's.  Launches go to torch's current stream; passes of one lane
    must follow each other on one stream, passes of different lanes may overlap."""

    def __init__(self, sess: Session):
        torch = sess.torch
        self.sess = sess
        self.x = torch.zeros_like(sess.x)
        self.y = torch.zeros_like(sess.y)
        self.workspace = torch.zeros(sess.info["workspace_bytes"] + 256, dtype=torch.uint8, device=sess.device)

    def set_input(self, x: np.ndarray):
        s = self.sess
        t = s.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(s.device)
        if s.in_fmt[1] == XENOS_NHWC:
            t = t.permute(0, 2, 3, 1)
        self.x.copy_(t)

    def run(self):
        s = self.sess
        xenos_run_with(s.plan, self.x.data_ptr(), self.y.data_ptr(), s._al(self.workspace), s.stream())

    def output(self) -> np.ndarray:
        s = self.sess
        s.torch.cuda.synchronize(s.device)
        y = self.y.float()
        if s.out_fmt[1] == XENOS_NHWC:
            y = y.permute(0, 3, 1, 2)
        return y.contiguous().cpu().numpy()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
