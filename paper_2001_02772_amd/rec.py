"""Thin binding of librec's C ABI (see include/rec.h): argument marshalling only.

Every step of the model runs in the library's HIP kernels.  PyTorch is used for
device memory (``torch.empty(..., device="cuda")``) and for the current stream,
nothing else.  There is no CPU fallback: a missing library or a non-zero status
raises.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "librec.so")
SOURCES = [os.path.join(_HERE, "csrc", f) for f in ("sls.hip", "fc.hip", "fc_fused.hip", "gemm_bf16.hip", "interact.hip", "model.hip", "sched.hip")]

OK, ERR_NULL, ERR_BAD_SHAPE, ERR_NEGATIVE_LENGTH, ERR_LENGTHS_MISMATCH, ERR_INDEX_RANGE, \
    ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_DEVICE = range(9)
F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_SIGMOID = 0, 1, 2
INTERACT_DOT, INTERACT_CONCAT = 0, 1

EXPORTS = (
    "rec_status_string", "rec_split_query",
    "rec_sls_workspace_bytes", "rec_sls_forward", "rec_sls_forward_static", "rec_sls_forward_offsets", "rec_sls_offsets",
    "rec_sls_validate",
    "rec_mlp_workspace_bytes", "rec_mlp_forward", "rec_f32_to_bf16",
    "rec_interact",
    "rec_model_padded_weight_bytes", "rec_model_create", "rec_model_prepare", "rec_model_destroy", "rec_model_workspace_bytes",
    "rec_model_forward",
    "rec_sched_query_service", "rec_sched_fifo_latencies", "rec_sched_percentile", "rec_sched_max_qps",
    "rec_sched_hill_climb", "rec_sched_two_tier_latencies", "rec_sched_two_tier_max_qps", "rec_serve_trace", "rec_serve_trace_many", "rec_model_forward_many",
    "rec_stream_pool_create", "rec_stream_pool_destroy", "rec_stream_pool_size", "rec_stream_pool_stream",
    "rec_stream_pool_synchronize",
)


class RecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


# Device code is built without packed fp32 arithmetic (v_pk_add/mul/fma_f32).  The switch is a target
# feature of the device compiler; hipcc hands it to its host pass too, which does not know it and says
# so ("not a recognized feature for this target") -- harmless.  tests/test_build_flags.py checks on the
# generated ISA that the device pass honours it.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    """Compile the HIP sources for gfx950 into librec.so next to this file."""
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-fPIC", "-shared", "-I" + os.path.join(_ROOT, "include"), "-pthread", "-o", LIB_PATH] + SOURCES
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    if verbose:
        print(" ".join(cmd))
        noise = "is not a recognized feature for this target"
        rest = [l for l in r.stderr.splitlines() if l.strip() and noise not in l and "warning generated" not in l
                and "warnings generated" not in l]
        print(f"hipcc: {r.stderr.count(noise)} host-pass notes about '-packed-fp32-ops' (expected), "
              f"{len(rest)} other lines of compiler output")
        for l in rest:
            print("  " + l)
    return LIB_PATH


_lib = None


class _PartialLibrary:
    """A library built from part of the sources (REC_LIB_PATH, e.g. the host-only sanitizer build of
    the serving functions): prototypes of entry points it lacks are set on placeholders and dropped."""

    class _Missing:
        restype = argtypes = None

    def __init__(self, cdll):
        self._cdll = cdll

    def __getattr__(self, name):
        try:
            return getattr(self._cdll, name)
        except AttributeError:
            if name.startswith("rec_"):
                return _PartialLibrary._Missing()
            raise


def lib():
    """Load librec.so (building it only if no built library exists).  REC_LIB_PATH names another build of
    the library to load instead (it may hold only some of the entry points)."""
    global _lib
    if _lib is not None:
        return _lib
    override = os.environ.get("REC_LIB_PATH")
    if override:
        L = _PartialLibrary(C.CDLL(override))
    else:
        if not os.path.exists(LIB_PATH):
            build_library()
        elif os.path.getmtime(LIB_PATH) < max(os.path.getmtime(f) for f in SOURCES + [os.path.join(_ROOT, "include", "rec.h")]):
            import warnings
            warnings.warn("librec.so is older than its sources: run __graft_entry__.build() (loading the existing build)",
                          RuntimeWarning)
        L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.rec_status_string.restype = C.c_char_p
    L.rec_status_string.argtypes = [C.c_int]
    L.rec_split_query.restype = i64
    L.rec_split_query.argtypes = [i64, i64, vp, vp]
    L.rec_sls_workspace_bytes.restype = sz
    L.rec_sls_workspace_bytes.argtypes = [i32, i32]
    L.rec_sls_forward.restype = C.c_int
    L.rec_sls_forward.argtypes = [vp, vp, i32, i32, vp, i64, vp, i32, vp, i64, i64, vp, sz, vp]
    L.rec_sls_forward_static.restype = C.c_int
    L.rec_sls_forward_static.argtypes = [vp, vp, i32, i32, vp, i64, vp, i32, vp, i64, i64, vp]
    L.rec_sls_forward_offsets.restype = C.c_int
    L.rec_sls_forward_offsets.argtypes = [vp, vp, i32, i32, vp, i64, vp, i32, vp, i64, i64, vp]
    L.rec_sls_offsets.restype = C.c_int
    L.rec_sls_offsets.argtypes = [vp, i64, vp, vp]
    L.rec_sls_validate.restype = C.c_int
    L.rec_sls_validate.argtypes = [vp, i32, vp, i64, vp, i32, vp, vp, vp, sz, vp]
    L.rec_mlp_workspace_bytes.restype = sz
    L.rec_mlp_workspace_bytes.argtypes = [vp, i32, i32, C.c_int]
    L.rec_mlp_forward.restype = C.c_int
    L.rec_mlp_forward.argtypes = [vp, vp, vp, i32, C.c_int, C.c_int, C.c_int, vp, i64, vp, i64, i32, vp, sz, vp]
    L.rec_f32_to_bf16.restype = C.c_int
    L.rec_f32_to_bf16.argtypes = [vp, vp, i64, vp]
    L.rec_interact.restype = C.c_int
    L.rec_interact.argtypes = [vp, i32, i32, i32, vp, i64, vp]
    L.rec_model_create.restype = C.c_int
    L.rec_model_create.argtypes = [vp, vp]
    L.rec_model_padded_weight_bytes.restype = sz
    L.rec_model_padded_weight_bytes.argtypes = [vp]
    L.rec_model_prepare.restype = C.c_int
    L.rec_model_prepare.argtypes = [vp, vp]
    L.rec_model_destroy.restype = None
    L.rec_model_destroy.argtypes = [vp]
    L.rec_model_workspace_bytes.restype = sz
    L.rec_model_workspace_bytes.argtypes = [vp, i32]
    L.rec_model_forward.restype = C.c_int
    L.rec_model_forward.argtypes = [vp, vp, vp, i64, vp, i32, vp, vp, sz, vp]
    L.rec_sched_query_service.restype = C.c_double
    L.rec_sched_query_service.argtypes = [i64, i64, vp]
    L.rec_sched_fifo_latencies.restype = C.c_int
    L.rec_sched_fifo_latencies.argtypes = [vp, vp, i64, vp]
    L.rec_sched_percentile.restype = C.c_double
    L.rec_sched_percentile.argtypes = [vp, i64, C.c_double]
    L.rec_sched_max_qps.restype = C.c_double
    L.rec_sched_max_qps.argtypes = [vp, vp, i64, C.c_double, C.c_double, i32]
    L.rec_sched_two_tier_latencies.restype = C.c_int
    L.rec_sched_two_tier_latencies.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp, i64, vp]
    L.rec_sched_two_tier_max_qps.restype = C.c_double
    L.rec_sched_two_tier_max_qps.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp, i64, C.c_double, C.c_double, i32]
    L.rec_sched_hill_climb.restype = i64
    L.rec_sched_hill_climb.argtypes = [vp, i64]
    L.rec_stream_pool_create.restype = C.c_int
    L.rec_stream_pool_create.argtypes = [i32, vp]
    L.rec_stream_pool_destroy.restype = None
    L.rec_stream_pool_destroy.argtypes = [vp]
    L.rec_stream_pool_size.restype = i32
    L.rec_stream_pool_size.argtypes = [vp]
    L.rec_stream_pool_stream.restype = vp
    L.rec_stream_pool_stream.argtypes = [vp, i32]
    L.rec_stream_pool_synchronize.restype = C.c_int
    L.rec_stream_pool_synchronize.argtypes = [vp]
    L.rec_model_forward_many.restype = C.c_int
    L.rec_model_forward_many.argtypes = [vp, vp, vp, i64, vp, vp, sz, i32]
    L.rec_serve_trace_many.restype = C.c_int
    L.rec_serve_trace_many.argtypes = [vp, vp, vp, vp, i64, vp, vp, sz, vp, i32, i32, vp]
    L.rec_serve_trace.restype = C.c_int
    L.rec_serve_trace.argtypes = [vp, vp, vp, vp, i64, vp, vp, sz, vp, vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    f = lib().rec_status_string
    return f(status).decode() if callable(f) else f"status {status}"      # (a partial build may lack the names)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise RecError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _workspace(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _host_i32(v):
    return np.ascontiguousarray(v, dtype=np.int32)


def _host_i64(v):
    return np.ascontiguousarray(v, dtype=np.int64)


def _ptr_array_host(tensors):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def split_query(n: int, batch: int):
    k = lib().rec_split_query(n, batch, None, None)
    if k < 0:
        raise RecError(ERR_BAD_SHAPE, "rec_split_query")
    start, count = np.empty(k, np.int64), np.empty(k, np.int64)
    lib().rec_split_query(n, batch, start.ctypes.data, count.ctypes.data)
    return list(zip(start.tolist(), count.tolist()))


class Tables:
    """T embedding tables on the device plus the device array of their base pointers."""

    def __init__(self, tables):
        self.tensors = list(tables)
        for t in self.tensors:
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.dim() == 2
        self.T = len(self.tensors)
        self.D = self.tensors[0].shape[1]
        self.rows = _host_i64([t.shape[0] for t in self.tensors])
        self.ptrs = torch.tensor([t.data_ptr() for t in self.tensors], dtype=torch.int64,
                                 device=self.tensors[0].device)


def sls_workspace_bytes(T: int, B: int) -> int:
    return lib().rec_sls_workspace_bytes(T, B)


def sls_forward(tables: Tables, indices, lengths, B: int, out=None, out_stride_b=None, out_stride_t=None,
                workspace=None):
    """E[b][t][:] = sum of the looked-up rows; returns fp32 [B][T][D] unless `out` is given."""
    T, D = tables.T, tables.D
    dev = tables.ptrs.device
    if out is None:
        out = torch.empty((B, T, D), dtype=torch.float32, device=dev)
        out_stride_b, out_stride_t = T * D, D
    if workspace is None:
        workspace = _workspace(sls_workspace_bytes(T, B), dev)
    st = lib().rec_sls_forward(_ptr(tables.ptrs), tables.rows.ctypes.data, T, D, _ptr(indices), indices.numel(),
                               _ptr(lengths), B, _ptr(out), out_stride_b, out_stride_t, _ptr(workspace),
                               workspace.numel(), _stream())
    _check(st, "rec_sls_forward")
    return out


SLS_STATIC_MAX_BAGS = 262144


def sls_forward_static(tables: Tables, indices, lengths, B: int, out=None, out_stride_b=None, out_stride_t=None):
    """rec_sls_forward_static: the same pooling with the offsets in the library's own static device array."""
    T, D = tables.T, tables.D
    if out is None:
        out = torch.empty((B, T, D), dtype=torch.float32, device=tables.ptrs.device)
        out_stride_b, out_stride_t = T * D, D
    st = lib().rec_sls_forward_static(_ptr(tables.ptrs), tables.rows.ctypes.data, T, D, _ptr(indices), indices.numel(),
                                      _ptr(lengths), B, _ptr(out), out_stride_b, out_stride_t, _stream())
    _check(st, "rec_sls_forward_static")
    return out


def sls_forward_offsets(tables: Tables, indices, offsets, B: int, out=None, out_stride_b=None, out_stride_t=None):
    """Pooling kernel alone, from precomputed int64 bag offsets."""
    T, D = tables.T, tables.D
    if out is None:
        out = torch.empty((B, T, D), dtype=torch.float32, device=tables.ptrs.device)
        out_stride_b, out_stride_t = T * D, D
    st = lib().rec_sls_forward_offsets(_ptr(tables.ptrs), tables.rows.ctypes.data, T, D, _ptr(indices),
                                       indices.numel(), _ptr(offsets), B, _ptr(out), out_stride_b, out_stride_t,
                                       _stream())
    _check(st, "rec_sls_forward_offsets")
    return out


def sls_offsets(lengths):
    n = lengths.numel()
    off = torch.empty(n + 1, dtype=torch.int64, device=lengths.device)
    _check(lib().rec_sls_offsets(_ptr(lengths), n, _ptr(off), _stream()), "rec_sls_offsets")
    return off


def sls_validate(rows, indices, lengths, B: int, workspace=None):
    """Returns (status, n_bad, first_bad); does not raise on data errors."""
    rows = _host_i64(rows)
    T = len(rows)
    if workspace is None:
        workspace = _workspace(sls_workspace_bytes(T, B), lengths.device)
    n_bad, first_bad = C.c_int64(0), C.c_int64(-1)
    st = lib().rec_sls_validate(rows.ctypes.data, T, _ptr(indices), indices.numel(), _ptr(lengths), B,
                                C.addressof(n_bad), C.addressof(first_bad), _ptr(workspace), workspace.numel(),
                                _stream())
    return st, n_bad.value, first_bad.value


def f32_to_bf16(src):
    """fp32 device tensor -> int16 tensor of bfloat16 bit patterns (round to nearest even)."""
    dst = torch.empty(src.shape, dtype=torch.int16, device=src.device)
    _check(lib().rec_f32_to_bf16(_ptr(src), _ptr(dst), src.numel(), _stream()), "rec_f32_to_bf16")
    return dst


def mlp_workspace_bytes(widths, B: int, wdtype: int) -> int:
    w = _host_i32(widths)
    return lib().rec_mlp_workspace_bytes(w.ctypes.data, len(w) - 1, B, wdtype)


def mlp_forward(W, bias, x, hidden_act=ACT_RELU, final_act=ACT_RELU, wdtype=F32, y=None, ldy=None, workspace=None):
    """W: list of device tensors [out][in] (fp32, or int16 bf16 patterns for BF16); x fp32 [B][in]."""
    widths = _host_i32([W[0].shape[1]] + [w.shape[0] for w in W])
    B = x.shape[0]
    if y is None:
        y = torch.empty((B, int(widths[-1])), dtype=torch.float32, device=x.device)
        ldy = int(widths[-1])
    if workspace is None:
        workspace = _workspace(mlp_workspace_bytes(widths, B, wdtype), x.device)
    Wp, bp = _ptr_array_host(W), _ptr_array_host(bias)
    st = lib().rec_mlp_forward(C.addressof(Wp), C.addressof(bp), widths.ctypes.data, len(W), wdtype, hidden_act,
                               final_act, _ptr(x), x.stride(0) if B else int(widths[0]), _ptr(y), ldy, B,
                               _ptr(workspace), workspace.numel(), _stream())
    _check(st, "rec_mlp_forward")
    return y


def interact(vecs, out=None, ldo=None):
    B, V, D = vecs.shape
    if out is None:
        ldo = D + V * (V - 1) // 2
        out = torch.empty((B, ldo), dtype=torch.float32, device=vecs.device)
    _check(lib().rec_interact(_ptr(vecs), B, V, D, _ptr(out), ldo, _stream()), "rec_interact")
    return out


class _ModelDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("D", C.c_int32), ("tables", C.c_void_p), ("rows", C.c_void_p),
                ("n_bottom", C.c_int32), ("bottom_widths", C.c_void_p), ("bottom_W", C.c_void_p),
                ("bottom_b", C.c_void_p),
                ("n_top", C.c_int32), ("top_widths", C.c_void_p), ("top_W", C.c_void_p), ("top_b", C.c_void_p),
                ("mlp_dtype", C.c_int), ("interaction", C.c_int),
                ("padded_weights", C.c_void_p), ("padded_weights_bytes", C.c_size_t)]


class Model:
    """Owns the device tensors of one model and the library handle that borrows them."""

    def __init__(self, tables: Tables, bottom_W, bottom_b, top_W, top_b, wdtype=F32, interaction=INTERACT_DOT,
                 dense_features: int | None = None, caller_padded_weights: bool = False):
        """interaction=INTERACT_CONCAT allows an empty bottom stack; then pass dense_features = F.
        caller_padded_weights: hand the library a buffer for its padded weight copy (host-only create
        + rec_model_prepare) instead of letting rec_model_create allocate it."""
        self.tables, self.wdtype, self.interaction = tables, wdtype, interaction
        self.bottom_W, self.bottom_b, self.top_W, self.top_b = list(bottom_W), list(bottom_b), list(top_W), list(top_b)
        self.bottom_widths = _host_i32([bottom_W[0].shape[1] if self.bottom_W else dense_features]
                                       + [w.shape[0] for w in bottom_W])
        self.top_widths = _host_i32([top_W[0].shape[1]] + [w.shape[0] for w in top_W])
        self.device = tables.ptrs.device
        arrays = [_ptr_array_host(a) for a in (self.bottom_W, self.bottom_b, self.top_W, self.top_b)]
        d = _ModelDesc(tables.T, tables.D, _ptr(tables.ptrs), tables.rows.ctypes.data,
                       len(self.bottom_W), self.bottom_widths.ctypes.data, C.addressof(arrays[0]), C.addressof(arrays[1]),
                       len(self.top_W), self.top_widths.ctypes.data, C.addressof(arrays[2]), C.addressof(arrays[3]),
                       wdtype, interaction, None, 0)
        self.padded_weight_bytes = lib().rec_model_padded_weight_bytes(C.addressof(d))
        self._padded = None
        if caller_padded_weights and self.padded_weight_bytes:
            self._padded = _workspace(self.padded_weight_bytes, self.device)
            d.padded_weights, d.padded_weights_bytes = _ptr(self._padded), self._padded.numel()
        h = C.c_void_p(0)
        _check(lib().rec_model_create(C.addressof(d), C.addressof(h)), "rec_model_create")
        self._h = h
        self._ws = None
        if self._padded is not None:
            _check(lib().rec_model_prepare(self._h, _stream()), "rec_model_prepare")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().rec_model_destroy(self._h)
            self._h = None

    __del__ = close

    def workspace_bytes(self, B: int) -> int:
        return lib().rec_model_workspace_bytes(self._h, B)

    def workspace(self, B: int) -> torch.Tensor:
        need = self.workspace_bytes(B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = _workspace(need, self.device)
        return self._ws

    def forward(self, dense, indices, lengths, B: int, prob=None, workspace=None):
        if prob is None:
            prob = torch.empty(B, dtype=torch.float32, device=self.device)
        if workspace is None:
            workspace = self.workspace(B)
        st = lib().rec_model_forward(self._h, _ptr(dense), _ptr(indices), indices.numel(), _ptr(lengths), B,
                                     _ptr(prob), _ptr(workspace), workspace.numel(), _stream())
        _check(st, "rec_model_forward")
        return prob


# ---- query serving and batch-size tuning (host arrays of float64) ----------------------------

def _host_f64(v):
    return np.ascontiguousarray(v, dtype=np.float64)


def sched_query_service(n: int, batch: int, table) -> float:
    table = _host_f64(table)
    assert table.size > batch
    return lib().rec_sched_query_service(n, batch, table.ctypes.data)


def sched_fifo_latencies(arrival, service):
    arrival, service = _host_f64(arrival), _host_f64(service)
    lat = np.empty_like(arrival)
    _check(lib().rec_sched_fifo_latencies(arrival.ctypes.data, service.ctypes.data, arrival.size, lat.ctypes.data),
           "rec_sched_fifo_latencies")
    return lat


def sched_percentile(x, p: float) -> float:
    x = _host_f64(x)
    return lib().rec_sched_percentile(x.ctypes.data, x.size, p)


def sched_max_qps(unit_arrival, service, p: float, sla: float, iters: int = 40) -> float:
    unit_arrival, service = _host_f64(unit_arrival), _host_f64(service)
    return lib().rec_sched_max_qps(unit_arrival.ctypes.data, service.ctypes.data, service.size, p, sla, iters)


def sched_hill_climb(qps) -> int:
    qps = _host_f64(qps)
    return lib().rec_sched_hill_climb(qps.ctypes.data, qps.size)


def sched_two_tier_latencies(arrival, size, tau: int, batch: int, c, k: int, g):
    arrival, size, c, g = _host_f64(arrival), _host_i64(size), _host_f64(c), _host_f64(g)
    assert c.size > batch
    lat = np.empty_like(arrival)
    _check(lib().rec_sched_two_tier_latencies(arrival.ctypes.data, size.ctypes.data, arrival.size, tau, batch, c.ctypes.data,
                                              k, g.ctypes.data, g.size - 1, lat.ctypes.data), "rec_sched_two_tier_latencies")
    return lat


def sched_two_tier_max_qps(unit_arrival, size, tau: int, batch: int, c, k: int, g, p: float, sla: float,
                           iters: int = 40) -> float:
    unit_arrival, size, c, g = _host_f64(unit_arrival), _host_i64(size), _host_f64(c), _host_f64(g)
    assert c.size > batch
    return lib().rec_sched_two_tier_max_qps(unit_arrival.ctypes.data, size.ctypes.data, size.size, tau, batch,
                                            c.ctypes.data, k, g.ctypes.data, g.size - 1, p, sla, iters)


class _Request(C.Structure):
    _fields_ = [("dense", C.c_void_p), ("indices", C.c_void_p), ("n_indices", C.c_int64), ("lengths", C.c_void_p),
                ("B", C.c_int32)]


class _PoolStream:
    def __init__(self, handle: int):
        self.cuda_stream = handle


class StreamPool:
    """Streams owned by the library (rec_stream_pool_*); .streams[i].cuda_stream is the raw handle."""

    def __init__(self, n: int):
        h = C.c_void_p(0)
        _check(lib().rec_stream_pool_create(n, C.addressof(h)), "rec_stream_pool_create")
        self._h = h
        self.streams = [_PoolStream(lib().rec_stream_pool_stream(h, i)) for i in range(lib().rec_stream_pool_size(h))]

    def synchronize(self):
        _check(lib().rec_stream_pool_synchronize(self._h), "rec_stream_pool_synchronize")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().rec_stream_pool_destroy(self._h)
            self._h = None

    __del__ = close


class ForwardMany:
    """Marshalled arguments of rec_model_forward_many for a fixed list of requests (device
    batches), outputs, streams and workspaces; launch() enqueues them all and returns at once."""

    def __init__(self, model: "Model", requests, probs, streams, workspaces=None):
        self.model, self.n, self.keep = model, len(requests), (requests, probs, streams)
        self.reqs = (_Request * max(self.n, 1))()
        for i, r in enumerate(requests):
            self.reqs[i] = _Request(_ptr(r.dense), _ptr(r.indices), r.indices.numel(), _ptr(r.lengths), r.B)
        self.probs = (C.c_void_p * max(self.n, 1))(*[_ptr(p) for p in probs])
        max_b = max([r.B for r in requests] + [1])
        need = model.workspace_bytes(max_b)
        self.ws = workspaces if workspaces is not None else [_workspace(need, model.device) for _ in streams]
        self.ws_bytes = min(w.numel() for w in self.ws)
        self.streams = (C.c_void_p * len(streams))(*[s.cuda_stream for s in streams])
        self.wsp = (C.c_void_p * len(streams))(*[_ptr(w) for w in self.ws])

    def launch(self):
        st = lib().rec_model_forward_many(self.model._h, C.addressof(self.reqs), C.addressof(self.probs), self.n,
                                          C.addressof(self.streams), C.addressof(self.wsp), self.ws_bytes,
                                          len(self.streams))
        _check(st, "rec_model_forward_many")


class ServeTrace:
    """Marshalled arguments of rec_serve_trace_many for a fixed list of queries (each a list of
    device batches); run(arrival_s) replays the trace and returns per-query latencies in seconds.
    streams: objects with .cuda_stream (None: torch's current stream)."""

    def __init__(self, model: "Model", queries, streams=None, spread_requests: bool = False):
        self.model, self.keep, self.spread = model, queries, int(spread_requests)
        flat = [r for q in queries for r in q]
        self.n = len(queries)
        self.reqs = (_Request * max(len(flat), 1))()
        for i, r in enumerate(flat):
            self.reqs[i] = _Request(_ptr(r.dense), _ptr(r.indices), r.indices.numel(), _ptr(r.lengths), r.B)
        self.first = _host_i64(np.concatenate([[0], np.cumsum([len(q) for q in queries])]))
        handles = [_stream()] if streams is None else [s.cuda_stream for s in streams]
        max_b = max([r.B for r in flat] + [1])
        self.ws_bytes = model.workspace_bytes(max_b)
        self.ws = [_workspace(self.ws_bytes, model.device) for _ in handles]
        self.prob = [torch.empty(max_b, dtype=torch.float32, device=model.device) for _ in handles]
        self.streams = (C.c_void_p * len(handles))(*handles)
        self.wsp = (C.c_void_p * len(handles))(*[_ptr(w) for w in self.ws])
        self.probp = (C.c_void_p * len(handles))(*[_ptr(p) for p in self.prob])

    def run(self, arrival_s):
        arrival_s = _host_f64(arrival_s)
        assert arrival_s.size == self.n
        lat = np.empty(self.n, dtype=np.float64)
        st = lib().rec_serve_trace_many(self.model._h, C.addressof(self.reqs), self.first.ctypes.data,
                                        arrival_s.ctypes.data, self.n, C.addressof(self.probp), C.addressof(self.wsp),
                                        self.ws_bytes, C.addressof(self.streams), len(self.streams), self.spread,
                                        lat.ctypes.data)
        _check(st, "rec_serve_trace_many")
        return lat


def serve_trace(model: "Model", queries, arrival_s, streams=None):
    """One replay; see ServeTrace."""
    return ServeTrace(model, queries, streams).run(arrival_s)
