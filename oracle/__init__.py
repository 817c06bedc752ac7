"""ORACLE -- test infrastructure only (see blas3_ref.c).

ctypes binding of the naive CPU level-3 BLAS definitions.  Only ``tests/``,
``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may import
this package; the GPU library never does.

Arrays are numpy arrays; the leading dimension is taken from the strides, the
storage order from which stride is the unit one.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libblas3_ref.so")
_lib = None

RowMajor, ColMajor = 101, 102
NoTrans, Trans, ConjTrans = 111, 112, 113
Upper, Lower = 121, 122
NonUnit, Unit = 131, 132
Left, Right = 141, 142


def build(force=False):
    """Compile blas3_ref.c with gcc (host only, OpenMP, no fast-math)."""
    src = os.path.join(_HERE, "blas3_ref.c")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(src)):
        return _LIB_PATH
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        # tests/test_oracle_mutants.py points this at deliberately broken builds to show that the pins
        # notice; nothing that judges the GPU path may run with it set (those callers check overridden())
        override = os.environ.get("ORACLE_LIB_OVERRIDE")
        if not override:
            build()
        lib = ctypes.CDLL(override or _LIB_PATH)
        ci, cd, vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        for n in ("ref_dgemm", "ref_sgemm"):
            getattr(lib, n).argtypes = [ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        for n in ("ref_dsyrk", "ref_ssyrk"):
            getattr(lib, n).argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, cd, vp, ci]
        for n in ("ref_dsyr2k", "ref_ssyr2k"):
            getattr(lib, n).argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        for n in ("ref_dsymm", "ref_ssymm"):
            getattr(lib, n).argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        for n in ("ref_dtrmm", "ref_strmm", "ref_dtrsm", "ref_strsm"):
            getattr(lib, n).argtypes = [ci, ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, ci]
        lib.ref_max_threads.restype = ci
        _lib = lib
    return _lib


def overridden():
    """True when the environment replaces the oracle's library (the mutant tests of the pins do)."""
    return bool(os.environ.get("ORACLE_LIB_OVERRIDE"))


def threads():
    """Number of OpenMP threads the oracle will use."""
    return _load().ref_max_threads()


def _layout(a, order):
    """(pointer, leading dimension) of a 2-D array stored in ``order``."""
    assert a.ndim == 2
    it = a.itemsize
    if a.size == 0:
        return a.ctypes.data, max(1, a.shape[0] if order == ColMajor else a.shape[1])
    if order == ColMajor:
        assert a.shape[0] <= 1 or a.strides[0] == it, "column-major array needs unit row stride"
        ld = a.strides[1] // it if a.shape[1] > 1 else max(1, a.shape[0])
        ld = max(ld, a.shape[0], 1)
    else:
        assert a.shape[1] <= 1 or a.strides[1] == it, "row-major array needs unit column stride"
        ld = a.strides[0] // it if a.shape[0] > 1 else max(1, a.shape[1])
        ld = max(ld, a.shape[1], 1)
    return a.ctypes.data, ld


def _prefix(*arrays):
    dt = arrays[0].dtype
    assert all(x.dtype == dt for x in arrays)
    return {np.dtype(np.float64): "d", np.dtype(np.float32): "s"}[dt]


def gemm(order, transa, transb, alpha, A, B, beta, C):
    """C <- alpha op(A) op(B) + beta C in place (Eq. 1a, un-tiled)."""
    M, N = C.shape
    K = A.shape[1] if transa == NoTrans else A.shape[0]
    pa, lda = _layout(A, order)
    pb, ldb = _layout(B, order)
    pc, ldc = _layout(C, order)
    fn = getattr(_load(), "ref_%sgemm" % _prefix(A, B, C))
    rc = fn(order, transa, transb, M, N, K, alpha, pa, lda, pb, ldb, beta, pc, ldc)
    if rc:
        raise ValueError("oracle gemm: rc=%d" % rc)
    return C


def syrk(order, uplo, trans, alpha, A, beta, C):
    """Triangle ``uplo`` of C <- alpha A A^T (or A^T A) + beta C in place (Eq. 1b)."""
    N = C.shape[0]
    K = A.shape[1] if trans == NoTrans else A.shape[0]
    pa, lda = _layout(A, order)
    pc, ldc = _layout(C, order)
    fn = getattr(_load(), "ref_%ssyrk" % _prefix(A, C))
    rc = fn(order, uplo, trans, N, K, alpha, pa, lda, beta, pc, ldc)
    if rc:
        raise ValueError("oracle syrk: rc=%d" % rc)
    return C


def syr2k(order, uplo, trans, alpha, A, B, beta, C):
    """Triangle ``uplo`` of C <- alpha (A B^T + B A^T) (or A^T B + B^T A) + beta C in place (Eq. 1e)."""
    N = C.shape[0]
    K = A.shape[1] if trans == NoTrans else A.shape[0]
    pa, lda = _layout(A, order)
    pb, ldb = _layout(B, order)
    pc, ldc = _layout(C, order)
    fn = getattr(_load(), "ref_%ssyr2k" % _prefix(A, B, C))
    rc = fn(order, uplo, trans, N, K, alpha, pa, lda, pb, ldb, beta, pc, ldc)
    if rc:
        raise ValueError("oracle syr2k: rc=%d" % rc)
    return C


def symm(order, side, uplo, alpha, A, B, beta, C):
    """C <- alpha A B + beta C (left) or alpha B A + beta C (right), A symmetric, one triangle stored (Eq. 1f)."""
    M, N = C.shape
    pa, lda = _layout(A, order)
    pb, ldb = _layout(B, order)
    pc, ldc = _layout(C, order)
    fn = getattr(_load(), "ref_%ssymm" % _prefix(A, B, C))
    rc = fn(order, side, uplo, M, N, alpha, pa, lda, pb, ldb, beta, pc, ldc)
    if rc:
        raise ValueError("oracle symm: rc=%d" % rc)
    return C


def trmm(order, side, uplo, transa, diag, alpha, A, B):
    """B <- alpha op(A) B (left) or alpha B op(A) (right) in place (Eq. 1d)."""
    M, N = B.shape
    pa, lda = _layout(A, order)
    pb, ldb = _layout(B, order)
    fn = getattr(_load(), "ref_%strmm" % _prefix(A, B))
    rc = fn(order, side, uplo, transa, diag, M, N, alpha, pa, lda, pb, ldb)
    if rc:
        raise ValueError("oracle trmm: rc=%d" % rc)
    return B


def trsm(order, side, uplo, transa, diag, alpha, A, B):
    """Solve op(A) X = alpha B (left) or X op(A) = alpha B (right); X overwrites B (Eq. 1c)."""
    M, N = B.shape
    pa, lda = _layout(A, order)
    pb, ldb = _layout(B, order)
    fn = getattr(_load(), "ref_%strsm" % _prefix(A, B))
    rc = fn(order, side, uplo, transa, diag, M, N, alpha, pa, lda, pb, ldb)
    if rc:
        raise ValueError("oracle trsm: rc=%d" % rc)
    return B
