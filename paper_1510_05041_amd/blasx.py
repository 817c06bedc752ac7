"""Thin Python binding of the C ABI in include/blasx.h (argument marshalling only).

Every step of the path -- task-ization, tile cache, scheduling, copies, kernels -- runs
inside ``libblasx.so``.  PyTorch is used for two things only: owning the HBM arena and the
HIP streams handed to ``blasx_init``, and allocating page-locked host matrices.

Matrix arguments may be numpy arrays, CPU torch tensors or raw integer addresses; they are
passed as host pointers, untouched.
"""
import ctypes
import os

import numpy as np

from . import _build

RowMajor, ColMajor = 101, 102
NoTrans, Trans, ConjTrans = 111, 112, 113
Upper, Lower = 121, 122
NonUnit, Unit = 131, 132
Left, Right = 141, 142


class Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "calls", "tasks", "tile_steps", "launches", "hits", "misses", "evictions", "refetches",
        "copies_h2d", "copies_d2h", "bytes_h2d", "bytes_d2h", "slot_waits", "peak_slots",
        "profiled_launches")] + [(n, ctypes.c_double) for n in ("flops", "t_total_s", "t_issue_s", "t_kernel_s")] + [
        ("invalidations", ctypes.c_uint64)] + [(n, ctypes.c_double) for n in (
            "t_wait_s", "t_kernel_busy_s", "t_copy_unoverlapped_s", "t_device_span_s")] + [("steps_general", ctypes.c_uint64), ("transfers_h2d", ctypes.c_uint64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class BlasxError(RuntimeError):
    def __init__(self, name, rc, text):
        super().__init__("%s failed: rc=%d (%s)" % (name, rc, text))
        self.rc = rc


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    if hasattr(x, "data_ptr"):          # torch tensor
        if getattr(x, "is_cuda", False):
            raise TypeError("matrices must be host memory")
        return x.data_ptr()
    raise TypeError("unsupported matrix argument: %r" % type(x))


_stream_cache = []


class Library:
    """One loaded copy of the C library (the product ``libblasx.so`` unless a path is given)."""

    def __init__(self, path=None):
        if path is None:
            # PyTorch owns the device memory and the streams and ships its own HIP runtime: load it
            # first so that this library binds to the same runtime instead of bringing a second one
            try:
                import torch  # noqa: F401
            except ImportError:
                pass
        path = path or _build.LIB_PATH
        if not os.path.exists(path):
            raise OSError("%s is not built: run __graft_entry__.build() (hipcc, gfx950) first" % path)
        self.path = path
        self._lib = lib = ctypes.CDLL(path)
        ci, cd, cf, vp, sz = ctypes.c_int, ctypes.c_double, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
        lib.blasx_dgemm.argtypes = [ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        lib.blasx_dgemm_noalloc.argtypes = lib.blasx_dgemm.argtypes
        lib.blasx_sgemm.argtypes = [ci, ci, ci, ci, ci, ci, cf, vp, ci, vp, ci, cf, vp, ci]
        lib.blasx_dsyrk.argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, cd, vp, ci]
        lib.blasx_ssyrk.argtypes = [ci, ci, ci, ci, ci, cf, vp, ci, cf, vp, ci]
        lib.blasx_dsyr2k.argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        lib.blasx_ssyr2k.argtypes = [ci, ci, ci, ci, ci, cf, vp, ci, vp, ci, cf, vp, ci]
        lib.blasx_dsymm.argtypes = [ci, ci, ci, ci, ci, cd, vp, ci, vp, ci, cd, vp, ci]
        lib.blasx_ssymm.argtypes = [ci, ci, ci, ci, ci, cf, vp, ci, vp, ci, cf, vp, ci]
        lib.blasx_dtrsm.argtypes = [ci, ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, ci]
        lib.blasx_strsm.argtypes = [ci, ci, ci, ci, ci, ci, ci, cf, vp, ci, vp, ci]
        lib.blasx_dtrmm.argtypes = [ci, ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, ci]
        lib.blasx_strmm.argtypes = [ci, ci, ci, ci, ci, ci, ci, cf, vp, ci, vp, ci]
        lib.blasx_init.argtypes = [vp, sz, ctypes.POINTER(vp), ci]
        lib.blasx_set_tile.argtypes = [ci]
        lib.blasx_set_streams.argtypes = [ci]
        lib.blasx_set_cache_bytes.argtypes = [sz]
        lib.blasx_set_option.argtypes = [ctypes.c_char_p, ctypes.c_long]
        lib.blasx_get_option.argtypes = [ctypes.c_char_p]
        lib.blasx_get_option.restype = ctypes.c_long
        lib.blasx_invalidate.argtypes = [vp, sz]
        lib.blasx_invalidate_matrix.argtypes = [vp, ci, ci, ci, ci]
        lib.blasx_host_alloc.argtypes = [sz]
        lib.blasx_host_alloc.restype = vp
        lib.blasx_host_free.argtypes = [vp]
        lib.blasx_get_stats.argtypes = [ctypes.POINTER(Stats)]
        lib.blasx_strerror.argtypes = [ci]
        lib.blasx_strerror.restype = ctypes.c_char_p
        lib.blasx_last_error.restype = ctypes.c_char_p
        self._keep = None

    # -- error handling ---------------------------------------------------------------
    def _check(self, name, rc):
        if rc != 0:
            text = self._lib.blasx_strerror(rc).decode()
            extra = self._lib.blasx_last_error().decode()
            raise BlasxError(name, rc, text + (": " + extra if extra and rc > 0 else ""))

    # -- run-time control ------------------------------------------------------------
    def init(self, arena_bytes, nstreams=4, arena_ptr=None, stream_ptrs=None):
        """blasx_init.  Without explicit pointers the arena is a torch uint8 CUDA tensor and the
        streams are torch.cuda.Stream objects (default priority); both are kept alive here."""
        keep = []
        if arena_ptr is None or stream_ptrs is None:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("no GPU visible: the HIP library cannot run")
            if arena_ptr is None:
                arena = torch.empty(int(arena_bytes), dtype=torch.uint8, device="cuda")
                keep.append(arena)
                arena_ptr = arena.data_ptr()
            if stream_ptrs is None:
                # the same streams for every init of the process: which hardware queue a new
                # stream lands on depends on what was created before it, and two roles that end
                # up sharing a queue serialise (measured: 68 -> 42 TFLOP/s); the first streams a
                # process creates get queues of their own
                # All four are made, and used once, at the first init of the process -- also when it asks
                # for fewer: a stream gets its hardware queue (the least loaded of the process's four) when
                # it is first used, so streams made or first used later, after other streams have come and
                # gone, can end up sharing a queue with the compute stream (measured: 72 -> 45 TFLOP/s)
                if not _stream_cache:
                    for _ in range(4):
                        st = torch.cuda.Stream()
                        torch.cuda.Event().record(st)
                        st.synchronize()
                        _stream_cache.append(st)
                streams = _stream_cache[:nstreams]
                keep.append(streams)
                stream_ptrs = [s.cuda_stream for s in streams]
        arr = (ctypes.c_void_p * nstreams)(*stream_ptrs)
        self._check("blasx_init", self._lib.blasx_init(arena_ptr, int(arena_bytes), arr, nstreams))
        self._keep = keep

    def arena_tensor(self):
        """The torch tensor that init() made for the tile arena (None when the caller supplied the memory)."""
        for k in self._keep or []:
            if hasattr(k, "data_ptr"):
                return k
        return None

    def init_raw(self, arena_bytes, nstreams=4):
        """blasx_init with NULL arena and streams: the library allocates its own."""
        self._check("blasx_init", self._lib.blasx_init(None, int(arena_bytes), None, nstreams))
        self._keep = None

    def shutdown(self):
        self._check("blasx_shutdown", self._lib.blasx_shutdown())
        self._keep = None

    def set_tile(self, T):
        self._check("blasx_set_tile", self._lib.blasx_set_tile(T))

    def set_streams(self, n):
        self._check("blasx_set_streams", self._lib.blasx_set_streams(n))

    def set_cache_bytes(self, cap):
        self._check("blasx_set_cache_bytes", self._lib.blasx_set_cache_bytes(int(cap)))

    def set_option(self, name, value):
        self._check("blasx_set_option(%s)" % name, self._lib.blasx_set_option(name.encode(), int(value)))

    def get_option(self, name):
        return self._lib.blasx_get_option(name.encode())

    def invalidate(self, a):
        """Forget cached tiles of the numpy array `a` (its whole address range)."""
        lo = a.ctypes.data
        self._check("blasx_invalidate", self._lib.blasx_invalidate(lo, int(a.nbytes if a.flags.contiguous else
                    sum((n - 1) * abs(st) for n, st in zip(a.shape, a.strides)) + a.itemsize)))

    def invalidate_matrix(self, A, ld, rows, cols, elem_size):
        self._check("blasx_invalidate_matrix", self._lib.blasx_invalidate_matrix(_ptr(A), ld, rows, cols, elem_size))

    def invalidate_all(self):
        self._check("blasx_invalidate_all", self._lib.blasx_invalidate_all())

    def host_alloc(self, nbytes):
        p = self._lib.blasx_host_alloc(int(nbytes))
        if not p:
            raise MemoryError("blasx_host_alloc(%d) failed" % nbytes)
        return p

    def host_free(self, ptr):
        self._check("blasx_host_free", self._lib.blasx_host_free(ptr))

    def get_stats(self):
        s = Stats()
        self._check("blasx_get_stats", self._lib.blasx_get_stats(ctypes.byref(s)))
        return s.as_dict()

    def reset_stats(self):
        self._check("blasx_reset_stats", self._lib.blasx_reset_stats())

    def strerror(self, rc):
        return self._lib.blasx_strerror(rc).decode()

    def last_error(self):
        return self._lib.blasx_last_error().decode()

    # -- level-3 routines: same argument lists as the C prototypes --------------------
    def dgemm(self, Order, TransA, TransB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        rc = self._lib.blasx_dgemm(Order, TransA, TransB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc)
        if check:
            self._check("blasx_dgemm", rc)
        return rc

    def dgemm_noalloc(self, Order, TransA, TransB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        rc = self._lib.blasx_dgemm_noalloc(Order, TransA, TransB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc)
        if check:
            self._check("blasx_dgemm_noalloc", rc)
        return rc

    def sgemm(self, Order, TransA, TransB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        rc = self._lib.blasx_sgemm(Order, TransA, TransB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc)
        if check:
            self._check("blasx_sgemm", rc)
        return rc

    def dsyrk(self, Order, Uplo, Trans_, N, K, alpha, A, lda, beta, C, ldc, check=True):
        rc = self._lib.blasx_dsyrk(Order, Uplo, Trans_, N, K, alpha, _ptr(A), lda, beta, _ptr(C), ldc)
        if check:
            self._check("blasx_dsyrk", rc)
        return rc

    def ssyrk(self, Order, Uplo, Trans_, N, K, alpha, A, lda, beta, C, ldc, check=True):
        rc = self._lib.blasx_ssyrk(Order, Uplo, Trans_, N, K, alpha, _ptr(A), lda, beta, _ptr(C), ldc)
        if check:
            self._check("blasx_ssyrk", rc)
        return rc

    def _syr2k(self, name, Order, Uplo, Trans_, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check):
        rc = getattr(self._lib, name)(Order, Uplo, Trans_, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc)
        if check:
            self._check(name, rc)
        return rc

    def dsyr2k(self, Order, Uplo, Trans_, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        return self._syr2k("blasx_dsyr2k", Order, Uplo, Trans_, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check)

    def ssyr2k(self, Order, Uplo, Trans_, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        return self._syr2k("blasx_ssyr2k", Order, Uplo, Trans_, N, K, alpha, A, lda, B, ldb, beta, C, ldc, check)

    def _symm(self, name, Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc, check):
        rc = getattr(self._lib, name)(Order, Side, Uplo, M, N, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc)
        if check:
            self._check(name, rc)
        return rc

    def dsymm(self, Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        return self._symm("blasx_dsymm", Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc, check)

    def ssymm(self, Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc, check=True):
        return self._symm("blasx_ssymm", Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc, check)

    def strsm(self, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb, check=True):
        rc = self._lib.blasx_strsm(Order, Side, Uplo, TransA, Diag, M, N, alpha, _ptr(A), lda, _ptr(B), ldb)
        if check:
            self._check("blasx_strsm", rc)
        return rc

    def strmm(self, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb, check=True):
        rc = self._lib.blasx_strmm(Order, Side, Uplo, TransA, Diag, M, N, alpha, _ptr(A), lda, _ptr(B), ldb)
        if check:
            self._check("blasx_strmm", rc)
        return rc

    def dtrsm(self, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb, check=True):
        rc = self._lib.blasx_dtrsm(Order, Side, Uplo, TransA, Diag, M, N, alpha, _ptr(A), lda, _ptr(B), ldb)
        if check:
            self._check("blasx_dtrsm", rc)
        return rc

    def dtrmm(self, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb, check=True):
        rc = self._lib.blasx_dtrmm(Order, Side, Uplo, TransA, Diag, M, N, alpha, _ptr(A), lda, _ptr(B), ldb)
        if check:
            self._check("blasx_dtrmm", rc)
        return rc


class HostBuffer:
    """Page-locked host memory from blasx_host_alloc, released when the object dies."""

    def __init__(self, lib, nbytes):
        self._lib = lib
        self.nbytes = int(nbytes)
        self.ptr = lib.host_alloc(max(self.nbytes, 8))

    def free(self):
        if self.ptr:
            self._lib.host_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pinned_matrix(rows, cols, dtype=np.float64, ld=None, lib=None):
    """Column-major rows x cols numpy view (leading dimension ld) of page-locked host memory.

    Returns (view, owner); keep ``owner`` alive as long as the view is used (``owner.free()``
    releases the memory at once).
    """
    lib = lib or default()
    ld = max(rows, 1) if ld is None else ld
    dt = np.dtype(dtype)
    count = int(ld) * int(max(cols, 1))
    owner = HostBuffer(lib, count * dt.itemsize)
    raw = (ctypes.c_char * (count * dt.itemsize)).from_address(owner.ptr)
    flat = np.frombuffer(raw, dtype=dt, count=count)
    view = flat.reshape((max(cols, 1), ld)).T[:rows, :cols]
    return view, owner


_default = None


def default():
    """The product library, loaded on first use; raises if it has not been built."""
    global _default
    if _default is None:
        _default = Library()
    return _default
