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
