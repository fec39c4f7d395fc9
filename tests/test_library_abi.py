"""CPU checks of the C-ABI boundary: the built library loads and exports every symbol that
include/gpgnn.h declares; the ctypes struct mirrors have the C layout's sizes."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "gpgnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gp_[a-z0-9_A-Z]+)\s*\(", text)))


@pytest.fixture(scope="module")
def cdll():
    import paper_2203_09697_amd as gp
    if not os.path.exists(gp.library_path()):
        from paper_2203_09697_amd import build
        build.build()
    return gp.load()


def test_every_declared_symbol_is_exported(cdll):
    import paper_2203_09697_amd as gp
    declared = _declared_symbols()
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(cdll, name), name
    assert sorted(gp.EXPORTED_SYMBOLS) == declared
    assert b"gfx950" in cdll.gp_version()


def test_struct_layouts():
    from paper_2203_09697_amd import binding as B
    assert C.sizeof(B._Dims) == 16 * 4
    assert C.sizeof(B._Graph) == 2 * 8 + 4 * 8 + 8 + 2 * 4 + 5 * 8
    assert C.sizeof(B._Basis) == 4 * 8
    assert C.sizeof(B._WeightsD) == (10 + 2 + 2 * 4 * B.GP_MAX_RES) * 8


def test_host_only_queries(cdll):
    n = C.c_size_t()
    assert cdll.gp_edges_workspace(C.c_int64(1000), C.byref(n)) == 0 and n.value >= 8008
    assert cdll.gp_edges_workspace(C.c_int64(-1), C.byref(n)) == -1
    assert cdll.gp_triplets_workspace(C.c_int64(10), C.c_int64(100), C.byref(n)) == 0 and n.value > 2800
    assert cdll.gp_triplets_workspace(C.c_int64(10), C.c_int64(100), None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2203_09697_amd import binding as B
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "_HERE", str(tmp_path))
    with pytest.raises(ImportError):
        B.load()
