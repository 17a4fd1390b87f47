"""CPU-only checks of the boundary: the library builds for gfx950, loads, and
exports exactly the entry points the header declares; host-only entry points
(status names, query splitting, size queries) behave."""
import os
import re

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rec():
    from paper_2001_02772_amd import rec as _rec
    if not os.path.exists(_rec.LIB_PATH):
        _rec.build_library()
    return _rec


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rec_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(rec):
    names = declared_functions()
    assert sorted(names) == sorted(rec.EXPORTS)
    L = rec.lib()
    for n in names:
        assert getattr(L, n) is not None, n


def test_status_strings(rec):
    assert rec.status_string(0) == "REC_OK"
    assert rec.status_string(5) == "REC_ERR_INDEX_RANGE"
    assert rec.status_string(99) == "REC_ERR_UNKNOWN"


def test_split_query_host(rec):
    for n in range(0, 130):
        for B in (1, 16, 64, 1024):
            assert rec.split_query(n, B) == oracle.split_query(n, B)
    with pytest.raises(rec.RecError):
        rec.split_query(5, 0)


def test_size_queries(rec):
    assert rec.sls_workspace_bytes(40, 1024) >= (40 * 1024 + 1) * 8
    assert rec.sls_workspace_bytes(40, 1024) % 256 == 0
    assert rec.sls_workspace_bytes(0, 4) == 0
    assert rec.mlp_workspace_bytes([884, 512, 128, 1], 1024, rec.F32) >= 2 * 1024 * 512 * 4
    assert rec.mlp_workspace_bytes([13, 1], 10, rec.F32) == 0


def test_serving_entry_points_reject_bad_arguments_on_the_host(rec):
    """Argument checks that return before any device call, so they run without a GPU."""
    import ctypes as C
    L = rec.lib()
    h = C.c_void_p(0)
    for n in (0, -1, 17):
        assert L.rec_stream_pool_create(n, C.addressof(h)) == rec.ERR_BAD_SHAPE and not h.value
    assert L.rec_stream_pool_create(4, None) == rec.ERR_NULL
    assert L.rec_stream_pool_size(None) == 0 and L.rec_stream_pool_stream(None, 0) is None
    assert L.rec_stream_pool_synchronize(None) == rec.ERR_NULL
    L.rec_stream_pool_destroy(None)
    assert L.rec_model_forward_many(None, None, None, 0, None, None, 0, 1) == rec.OK         # nothing to do
    assert L.rec_model_forward_many(None, None, None, 3, None, None, 0, 0) == rec.ERR_BAD_SHAPE
    assert L.rec_model_forward_many(None, None, None, 3, None, None, 0, 2) == rec.ERR_NULL
    assert L.rec_serve_trace_many(None, None, None, None, 0, None, None, 0, None, 1, 0, None) == rec.OK
    assert L.rec_serve_trace_many(None, None, None, None, 2, None, None, 0, None, 0, 1, None) == rec.ERR_BAD_SHAPE
    assert L.rec_serve_trace_many(None, None, None, None, 2, None, None, 0, None, 1, 1, None) == rec.ERR_NULL
    assert L.rec_serve_trace(None, None, None, None, -1, None, None, 0, None, None) == rec.ERR_BAD_SHAPE


def test_header_is_c99_and_host_entry_points_work_from_c(rec, tmp_path):
    """tests/c_abi_host.c includes include/rec.h as C99 and calls the host-side entry points."""
    import subprocess
    exe = str(tmp_path / "c_abi_host")
    libdir = os.path.dirname(rec.LIB_PATH)
    cc = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I" + os.path.join(ROOT, "include"),
          os.path.join(ROOT, "tests", "c_abi_host.c"), "-o", exe, "-L" + libdir, "-l:librec.so", "-lm",
          "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cc, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "c abi ok" in r.stdout, r.stdout + r.stderr


def test_mlp_workspace_never_shrinks_with_the_batch(rec):
    """A workspace sized for the largest batch serves every smaller one (the serving entry points rely on it)."""
    for widths, dt in (([2560, 1024, 256, 32], rec.BF16), ([87, 512, 256, 1], rec.BF16), ([2048, 1024, 512, 256, 1], rec.BF16),
                       ([884, 512, 128, 1], rec.F32), ([896, 512, 128, 1], rec.F32)):
        top = rec.mlp_workspace_bytes(widths, 4096, dt)
        prev = 0
        for B in list(range(1, 300)) + list(range(300, 4097, 7)) + [4096]:
            b = rec.mlp_workspace_bytes(widths, B, dt)
            assert prev <= b <= top, (widths, B, prev, b, top)
            prev = b


def test_host_only_model_create_with_a_caller_buffer(rec):
    """With a caller-provided padded-weights buffer rec_model_create touches no device (it works here, without
    one), and the forward refuses to run until rec_model_prepare has filled the buffer."""
    import ctypes as C
    import numpy as np
    L = rec.lib()
    fake = 0x7f0000001000                                   # never dereferenced on the host; 256-byte aligned
    bw, tw = np.array([13, 32], np.int32), np.array([87, 64, 1], np.int32)
    rows = np.full(10, 1000, np.int64)
    ptrs = (C.c_void_p * 2)(fake, fake)
    d = rec._ModelDesc(10, 32, fake, rows.ctypes.data, 1, bw.ctypes.data, C.addressof(ptrs), C.addressof(ptrs),
                       2, tw.ctypes.data, C.addressof(ptrs), C.addressof(ptrs), rec.F32, rec.INTERACT_DOT, None, 0)
    need = L.rec_model_padded_weight_bytes(C.addressof(d))
    assert need == 64 * 88 * 4
    h = C.c_void_p(0)
    d.padded_weights, d.padded_weights_bytes = fake, need - 1
    assert L.rec_model_create(C.addressof(d), C.addressof(h)) == rec.ERR_WORKSPACE and not h.value
    d.padded_weights, d.padded_weights_bytes = fake + 8, need
    assert L.rec_model_create(C.addressof(d), C.addressof(h)) == rec.ERR_WORKSPACE and not h.value      # misaligned
    d.padded_weights, d.padded_weights_bytes = fake, need
    assert L.rec_model_create(C.addressof(d), C.addressof(h)) == rec.OK and h.value
    assert L.rec_model_workspace_bytes(h, 256) > 0
    assert L.rec_model_forward(h, fake, fake, 0, fake, 4, fake, fake, 1 << 30, None) == rec.ERR_BAD_SHAPE   # not prepared
    L.rec_model_destroy(h)
