"""Seeded synthetic inputs (shared by the oracle side and the GPU side of a test).

Only random-number filling lives here; none of the method's arithmetic does.
The C routines in ``synth.c`` are built into ``libsynth.so`` beside this file;
``fill`` etc. write straight into a caller-supplied buffer (a numpy array or a
pinned torch tensor viewed as numpy), so multi-gigabyte matrices are generated
in place with all host cores.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_lib = None

MAT_A, MAT_B, MAT_C = 0, 1, 2


def build(force=False):
    """Compile synth.c with gcc (host only)."""
    src = os.path.join(_HERE, "synth.c")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(src)):
        return _LIB_PATH
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        i64, u64, ci = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
        for name in ("synth_fill_f64", "synth_fill_f32", "synth_fill_int_f64", "synth_fill_int_f32"):
            getattr(lib, name).argtypes = [ctypes.c_void_p, i64, i64, i64, u64, ci]
            getattr(lib, name).restype = None
        for name in ("synth_dominant_diag_f64", "synth_dominant_diag_f32"):
            getattr(lib, name).argtypes = [ctypes.c_void_p, i64, i64, u64, ci]
            getattr(lib, name).restype = None
        for name in ("synth_block_f64", "synth_block_f32"):
            getattr(lib, name).argtypes = [ctypes.c_void_p, i64, i64, i64, i64, i64, i64, u64, ci]
            getattr(lib, name).restype = None
        lib.synth_element.argtypes = [u64, ci, i64, i64, i64]
        lib.synth_element.restype = ctypes.c_double
        _lib = lib
    return _lib


def _check_colmajor(a):
    if a.ndim != 2 or not a.flags["F_CONTIGUOUS"] and not (a.strides[0] == a.itemsize):
        raise ValueError("expected a column-major 2-D array (unit stride along rows)")
    return a.strides[1] // a.itemsize if a.shape[1] > 1 else max(1, a.shape[0])


def fill(a, seed, mat, integers=False):
    """Fill column-major array ``a`` (float64 or float32) in place; returns ``a``."""
    lib = _load()
    ld = _check_colmajor(a)
    rows, cols = a.shape
    kind = {np.dtype(np.float64): "f64", np.dtype(np.float32): "f32"}[a.dtype]
    fn = getattr(lib, ("synth_fill_int_" if integers else "synth_fill_") + kind)
    fn(a.ctypes.data, rows, cols, ld, seed, mat)
    return a


def matrix(rows, cols, seed, mat, dtype=np.float64, ld=None, integers=False):
    """New column-major rows x cols matrix (optionally padded to leading dimension ld)."""
    ld = rows if ld is None else ld
    buf = np.zeros((max(ld, 1), cols), dtype=dtype, order="F")
    a = buf[:rows, :]
    if rows and cols:
        fill(a, seed, mat, integers=integers)
    return a


def dominant_diag(a, seed, mat):
    """Set diag(a) = n + uniform[0,1) in place (square column-major ``a``)."""
    lib = _load()
    ld = _check_colmajor(a)
    n = a.shape[0]
    assert a.shape[1] == n
    kind = {np.dtype(np.float64): "f64", np.dtype(np.float32): "f32"}[a.dtype]
    getattr(lib, "synth_dominant_diag_" + kind)(a.ctypes.data, n, ld, seed, mat)
    return a


def block(seed, mat, rows, r0, c0, nr, nc, dtype=np.float64):
    """The nr x nc block at (r0, c0) of the matrix ``fill`` makes for a ``rows``-row array, regenerated on its own."""
    out = np.zeros((nr, nc), dtype=dtype, order="F")
    kind = {np.dtype(np.float64): "f64", np.dtype(np.float32): "f32"}[out.dtype]
    if nr and nc:
        getattr(_load(), "synth_block_" + kind)(out.ctypes.data, r0, c0, nr, nc, nr, rows, seed, mat)
    return out


def element(seed, mat, i, j, rows):
    """Element (i, j) of the uniform[-1,1) stream, regenerated on its own."""
    return _load().synth_element(seed, mat, i, j, rows)


def sample_tiles(nt_rows, nt_cols, count, seed):
    """``count`` distinct (i, j) tile indices (all of them if fewer exist)."""
    total = nt_rows * nt_cols
    rng = np.random.default_rng(seed)
    if total <= count:
        flat = np.arange(total)
    else:
        flat = rng.choice(total, size=count, replace=False)
    return [(int(f) // nt_cols, int(f) % nt_cols) for f in flat]
