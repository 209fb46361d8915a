"""The C-ABI library loads on a machine without a GPU and exports every symbol the header
declares; argument validation that needs no device is exercised here too."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "polydl.h")
LIB = os.path.join(ROOT, "paper_2006_02230_amd", "libpolydl.so")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(polydl_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libpolydl.so is not built (run __graft_entry__.build())")
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "polydl_conv2d_fwd" in names and "polydl_sgemm" in names
    for n in names:
        assert hasattr(lib, n), n


def test_argument_validation_without_device(lib):
    z, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    assert lib.polydl_sgemm(0, 1, 1, one, one, one, z) == -2
    assert lib.polydl_sgemm(2, 2, 2, z, one, one, z) == -1
    lib.polydl_sgemm_ex.argtypes = [ctypes.c_int] * 3 + [ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                                         ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.polydl_sgemm_ex(2, 0, 2, 1.0, one, one, 1.0, one, z) == -2
    assert lib.polydl_sgemm_ex(2, 2, 2, 1.0, one, one, 0.0, z, z) == -1
    assert lib.polydl_conv2d_fwd(1, 1, 2, 2, 1, 3, 3, 1, 0, one, one, z, one, 0, z) == -2
    assert lib.polydl_conv2d_fwd(1, 1, 4, 4, 1, 3, 3, 1, 1, z, one, z, one, 0, z) == -1
    lib.polydl_status_string.restype = ctypes.c_char_p
    assert lib.polydl_status_string(0) == b"ok"
    assert lib.polydl_status_string(-2) == b"bad dimension"


def test_variant_table(lib):
    import paper_2006_02230_amd as p
    vs = p.variants(0)
    assert len(vs) >= 4 and len(vs) > len(p.variants(1))
    assert {v.algo for v in vs} == {0, 1, 2}
    for v in vs:
        assert v.bm % v.wm == 0 and v.bn % v.wn == 0 and v.bk % 8 == 0
    bad = p.TileCfg(17, 64, 16, 32, 32, 1, 0, 0, 0, 0)
    assert lib.polydl_set_tile_override(ctypes.byref(bad)) == -3
    assert lib.polydl_set_tile_override(None) == 0
