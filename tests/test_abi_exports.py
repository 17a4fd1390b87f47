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
