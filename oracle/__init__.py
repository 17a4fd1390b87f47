"""ctypes binding of the CPU oracle (``rec_oracle.c``).  TEST INFRASTRUCTURE ONLY:
imported by tests, the smoke check and the benchmark's CPU-baseline leg; the
product package never imports it.  Arguments are NumPy arrays; every function
returns new arrays."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rec_oracle.c")
_LIB = os.path.join(_HERE, "librec_oracle.so")

OK, ERR_NULL, ERR_BAD_SHAPE, ERR_NEGATIVE_LENGTH, ERR_LENGTHS_MISMATCH, ERR_INDEX_RANGE = range(6)
ACT_NONE, ACT_RELU, ACT_SIGMOID = range(3)


def build(force: bool = False) -> str:
    override = os.environ.get("REC_ORACLE_LIB")   # lets a test load a deliberately broken copy
    if override:
        return override
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_bf16_round.restype = C.c_float
        _lib.orc_bf16_round.argtypes = [C.c_float]
        _lib.orc_split_query.restype = C.c_int64
        _lib.orc_split_query.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.orc_query_service.restype = C.c_double
        _lib.orc_query_service.argtypes = [C.c_int64, C.c_int64, C.c_void_p]
        _lib.orc_fifo_latencies.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        _lib.orc_percentile.restype = C.c_double
        _lib.orc_percentile.argtypes = [C.c_void_p, C.c_int64, C.c_double]
        _lib.orc_max_qps.restype = C.c_double
        _lib.orc_max_qps.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_double, C.c_int32]
        _lib.orc_hill_climb.restype = C.c_int64
        _lib.orc_hill_climb.argtypes = [C.c_void_p, C.c_int64]
    return _lib


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(n))


def get_threads() -> int:
    return lib().orc_get_threads()


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr_array(arrs):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def bf16_round(x):
    x = _f32(x)
    out = np.empty_like(x)
    lib().orc_bf16_round_array(_p(x), _p(out), C.c_int64(x.size))
    return out


def validate(rows, indices, lengths, B):
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    indices, lengths = _i32(indices), _i32(lengths)
    n_bad, first_bad = C.c_int64(0), C.c_int64(0)
    st = lib().orc_validate(_p(rows), C.c_int32(len(rows)), _p(indices), C.c_int64(indices.size),
                            _p(lengths), C.c_int32(B), C.byref(n_bad), C.byref(first_bad))
    return st, n_bad.value, first_bad.value


def offsets(lengths):
    lengths = _i32(lengths)
    off = np.empty(lengths.size + 1, dtype=np.int64)
    lib().orc_offsets(_p(lengths), C.c_int64(lengths.size), _p(off))
    return off


def sls(tables, indices, lengths, B, extra=False):
    """tables: list of fp32 [R_t][D].  Returns E fp32 [B][T][D]
    (and, with extra=True, the fp32 in-order sum and the fp64 sum of |x|)."""
    tables = [_f32(t) for t in tables]
    T, D = len(tables), tables[0].shape[1]
    indices = _i32(indices)
    off = offsets(lengths)
    assert off.size == T * B + 1
    out = np.zeros((B, T, D), dtype=np.float32)
    seq = np.zeros((B, T, D), dtype=np.float32) if extra else None
    aabs = np.zeros((B, T, D), dtype=np.float64) if extra else None
    lib().orc_sls(_ptr_array(tables), C.c_int32(T), C.c_int32(D), _p(indices), _p(off), C.c_int32(B),
                  _p(out), C.c_int64(T * D), C.c_int64(D),
                  _p(seq) if extra else None, _p(aabs) if extra else None)
    return (out, seq, aabs) if extra else out


def fc(x, W, bias, act, bf16=False):
    x, W, bias = _f32(x), _f32(W), _f32(bias)
    B, n_in = x.shape
    n_out = W.shape[0]
    assert W.shape == (n_out, n_in) and bias.shape == (n_out,)
    y = np.empty((B, n_out), dtype=np.float32)
    lib().orc_fc(_p(x), C.c_int64(n_in), _p(W), _p(bias), C.c_int32(B), C.c_int32(n_in),
                 C.c_int32(n_out), C.c_int32(act), C.c_int32(int(bf16)), _p(y), C.c_int64(n_out))
    return y


def mlp(x, Ws, biases, hidden_act, final_act, bf16=False):
    x = _f32(x)
    Ws, biases = [_f32(w) for w in Ws], [_f32(b) for b in biases]
    widths = np.array([Ws[0].shape[1]] + [w.shape[0] for w in Ws], dtype=np.int32)
    B = x.shape[0]
    y = np.empty((B, int(widths[-1])), dtype=np.float32)
    lib().orc_mlp(_ptr_array(Ws), _ptr_array(biases), _p(widths), C.c_int32(len(Ws)),
                  C.c_int32(int(bf16)), C.c_int32(hidden_act), C.c_int32(final_act), _p(x),
                  C.c_int64(x.shape[1]), _p(y), C.c_int64(y.shape[1]), C.c_int32(B))
    return y


def interact(vecs):
    vecs = _f32(vecs)
    B, V, D = vecs.shape
    out = np.empty((B, D + V * (V - 1) // 2), dtype=np.float32)
    lib().orc_interact(_p(vecs), C.c_int32(B), C.c_int32(V), C.c_int32(D), _p(out),
                       C.c_int64(out.shape[1]))
    return out


def model_forward(tables, Wb, bb, Wt, bt, dense, indices, lengths, bf16=False, concat=False):
    """Returns (status, prob fp32 [B]).  concat=True: the concatenating model (Wb may be empty)."""
    tables = [_f32(t) for t in tables]
    T, D = len(tables), tables[0].shape[1]
    rows = np.array([t.shape[0] for t in tables], dtype=np.int64)
    Wb, bb = [_f32(w) for w in Wb], [_f32(b) for b in bb]
    Wt, bt = [_f32(w) for w in Wt], [_f32(b) for b in bt]
    dense = _f32(dense)
    wb = np.array([Wb[0].shape[1] if Wb else dense.shape[1]] + [w.shape[0] for w in Wb], dtype=np.int32)
    wt = np.array([Wt[0].shape[1]] + [w.shape[0] for w in Wt], dtype=np.int32)
    dense, indices, lengths = _f32(dense), _i32(indices), _i32(lengths)
    B = dense.shape[0]
    prob = np.zeros(B, dtype=np.float32)
    fn = lib().orc_model_forward_concat if concat else lib().orc_model_forward
    st = fn(
        _ptr_array(tables), _p(rows), C.c_int32(T), C.c_int32(D),
        _ptr_array(Wb), _ptr_array(bb), _p(wb), C.c_int32(len(Wb)),
        _ptr_array(Wt), _ptr_array(bt), _p(wt), C.c_int32(len(Wt)),
        C.c_int32(int(bf16)), _p(dense), _p(indices), C.c_int64(indices.size), _p(lengths),
        C.c_int32(B), _p(prob))
    return st, prob


def split_query(n: int, Bsz: int):
    k = lib().orc_split_query(n, Bsz, None, None)
    start, count = np.empty(k, dtype=np.int64), np.empty(k, dtype=np.int64)
    lib().orc_split_query(n, Bsz, _p(start), _p(count))
    return list(zip(start.tolist(), count.tolist()))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def query_service(n: int, B: int, table) -> float:
    """table[b] = seconds for one request of b items (index 0 unused)."""
    table = _f64(table)
    assert table.size > B
    return lib().orc_query_service(n, B, _p(table))


def fifo_latencies(arrival, service):
    arrival, service = _f64(arrival), _f64(service)
    lat = np.empty_like(arrival)
    lib().orc_fifo_latencies(_p(arrival), _p(service), arrival.size, _p(lat))
    return lat


def percentile(x, p: float) -> float:
    x = _f64(x)
    return lib().orc_percentile(_p(x), x.size, p)


def max_qps(unit_arrival, service, p: float, sla: float, iters: int = 40) -> float:
    unit_arrival, service = _f64(unit_arrival), _f64(service)
    return lib().orc_max_qps(_p(unit_arrival), _p(service), service.size, p, sla, iters)


def hill_climb(qps) -> int:
    qps = _f64(qps)
    return lib().orc_hill_climb(_p(qps), qps.size)


def _i64(v):
    return np.ascontiguousarray(v, dtype=np.int64)


def two_tier_latencies(arrival, size, tau: int, B: int, c, k: int, g):
    """Latencies with queries of size >= tau on the accelerator (service g[size]) and the rest cut
    into requests of B on k CPU workers (service c[b])."""
    arrival, size, c, g = _f64(arrival), _i64(size), _f64(c), _f64(g)
    assert c.size > B and g.size > (size.max() if size.size else 0)
    lat = np.empty_like(arrival)
    lib().orc_two_tier_latencies(_p(arrival), _p(size), C.c_int64(arrival.size), C.c_int64(tau), C.c_int64(B), _p(c),
                                 C.c_int32(k), _p(g), _p(lat))
    return lat


def two_tier_max_qps(unit_arrival, size, tau: int, B: int, c, k: int, g, p: float, sla: float, iters: int = 40):
    unit_arrival, size, c, g = _f64(unit_arrival), _i64(size), _f64(c), _f64(g)
    f = lib().orc_two_tier_max_qps
    f.restype = C.c_double
    return f(_p(unit_arrival), _p(size), C.c_int64(size.size), C.c_int64(tau), C.c_int64(B), _p(c), C.c_int32(k), _p(g),
             C.c_double(p), C.c_double(sla), C.c_int32(iters))

