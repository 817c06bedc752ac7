"""The C-ABI library loads without a GPU and exports every symbol include/blasx.h declares."""
import ctypes
import os
import re

from paper_1510_05041_amd import _build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "blasx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(blasx_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = declared_symbols()
    for must in ("blasx_dgemm", "blasx_sgemm", "blasx_dsyrk", "blasx_dtrsm", "blasx_dtrmm", "blasx_init",
                 "blasx_shutdown", "blasx_set_tile", "blasx_set_cache_bytes", "blasx_get_stats", "blasx_strerror"):
        assert must in names


def test_product_library_exports_every_declared_symbol():
    """No compute call here: loading and symbol lookup only (the build step made the library)."""
    assert os.path.exists(_build.LIB_PATH), "run __graft_entry__.build() first"
    lib = ctypes.CDLL(_build.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    lib.blasx_strerror.restype = ctypes.c_char_p
    assert lib.blasx_strerror(2) == b"tile cache too small"
    # without blasx_init every routine refuses to run rather than falling back to anything
    a = (ctypes.c_double * 4)()
    lib.blasx_dgemm.argtypes = [ctypes.c_int] * 6 + [ctypes.c_double, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                                      ctypes.c_int, ctypes.c_double, ctypes.c_void_p, ctypes.c_int]
    assert lib.blasx_dgemm(102, 111, 111, 2, 2, 2, 1.0, a, 2, a, 2, 0.0, a, 2) == 1   # BLASX_ERR_NOT_INITIALIZED


def test_test_double_exports_the_same_symbols():
    lib = ctypes.CDLL(_build.build_sim())
    for name in declared_symbols():
        assert hasattr(lib, name), name
