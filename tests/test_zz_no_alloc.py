"""The allocation-free entry point blasx_dgemm_noalloc against blasx_dgemm, through the C ABI, on the device.

Two calls in a row share the statically allocated tile arena, the second on a smaller problem than the first
(so it finds the first one's tiles in every slot it uses); each result is compared with the existing entry
point's on the same inputs -- bit for bit on integer inputs, to the normwise 1e-13 gate and the elementwise
bound on uniform ones -- and sizes beyond the stated maximum are refused before anything is computed.
"""
import numpy as np
import pytest

import synth
from paper_1510_05041_amd import blasx

pytestmark = pytest.mark.gpu

U64 = 2.0 ** -53


def _norms(x, axis):
    x = np.asarray(x, dtype=np.float64)
    return np.sqrt(np.einsum("ij,ij->i" if axis == 1 else "ij,ij->j", x, x))


def _pinned(lib, rows, cols, seed, mat, integers=False):
    a, owner = blasx.pinned_matrix(rows, cols, lib=lib)
    synth.fill(a, seed, mat, integers=integers)
    return a, owner


def _pair(lib, ta, tb, M, N, K, alpha, beta, seed, integers):
    """The same problem through both entry points; returns (no-alloc result, existing entry point's result, A, B, C0)."""
    A, ka = _pinned(lib, *((M, K) if ta == blasx.NoTrans else (K, M)), seed, 0, integers)
    B, kb = _pinned(lib, *((K, N) if tb == blasx.NoTrans else (N, K)), seed, 1, integers)
    C1, k1 = _pinned(lib, M, N, seed, 2, integers)
    C2, k2 = _pinned(lib, M, N, seed, 2, integers)
    C0 = np.array(C1, order="F")
    lib.dgemm_noalloc(blasx.ColMajor, ta, tb, M, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C1, M)
    lib.dgemm(blasx.ColMajor, ta, tb, M, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C2, M)
    return np.array(C1), np.array(C2), np.array(A), np.array(B), C0, (ka, kb, k1, k2)


def test_noalloc_entry_point_matches_blasx_dgemm_on_two_calls_in_a_row_the_second_smaller():
    import torch
    assert torch.cuda.is_available()
    lib = blasx.default()
    lib.init(int(1.0 * 2 ** 30), nstreams=4)
    lib.set_tile(512)
    lib.set_cache_bytes(0)
    for k, v in dict(group=0, kchain=0, wide=11, depth=6, rs=32, profile=0, persist=0, ramp=0, priority=1, shells=1, sb_rows=4, sb_cols=4).items():
        lib.set_option(k, v)
    try:
        # first call: 5 x 4 output tiles with a ragged edge and 5 k-tiles, uniform data, transposed A
        got, want, A, B, C0, keep1 = _pair(lib, blasx.Trans, blasx.NoTrans, 2500, 1900, 2304, -0.75, 0.5, 60, False)
        assert np.all(np.isfinite(got))
        err = np.linalg.norm(got - want) / np.linalg.norm(want)
        assert err < 1e-13, err
        # both results carry their own rounding: twice the elementwise bound of one
        bound = 2 * (8 * U64 * 0.75 * np.outer(_norms(A, 0), _norms(B, 0)) + 4 * U64 * np.abs(0.5 * C0))
        assert np.all(np.abs(got - want) <= bound)
        # second call, smaller, integers: bit for bit, although every slot still holds the first call's tiles
        got2, want2, A2, B2, C02, keep2 = _pair(lib, blasx.NoTrans, blasx.Trans, 1024, 700, 1536, 2.0, -1.0, 61, True)
        assert np.array_equal(got2, want2)
        assert np.array_equal(got2, 2.0 * (A2 @ B2.T) - C02)
        # a third, uniform again and smaller still, beta = 0 over NaN: nothing of the old contents may show
        A3, k3a = _pinned(lib, 600, 520, 62, 0)
        B3, k3b = _pinned(lib, 520, 300, 62, 1)
        C3, k3c = blasx.pinned_matrix(600, 300, lib=lib)
        C4, k3d = blasx.pinned_matrix(600, 300, lib=lib)
        C3[...] = np.nan
        C4[...] = np.nan
        lib.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 600, 300, 520, 1.0, A3, 600, B3, 520, 0.0, C3, 600)
        lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 600, 300, 520, 1.0, A3, 600, B3, 520, 0.0, C4, 600)
        assert np.all(np.isfinite(np.asarray(C3)))
        assert np.linalg.norm(np.asarray(C3) - np.asarray(C4)) / np.linalg.norm(np.asarray(C4)) < 1e-13
        assert np.all(np.abs(np.asarray(C3) - np.asarray(C4)) <= 2 * 8 * U64 * np.outer(_norms(A3, 1), _norms(B3, 0)))

        # beyond the stated maximum: refused with its own code, nothing written
        n = 4096                                        # 3 * 8 * 8 = 192 tiles of 512 x 512 against 128 slots
        Ab, kba = blasx.pinned_matrix(n, n, lib=lib)
        Cb, kbc = blasx.pinned_matrix(n, n, lib=lib)
        Ab[...] = 1.0
        Cb[...] = 7.0
        rc = lib.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, Ab, n, Ab, n, 0.0, Cb, n, check=False)
        assert rc == 7 and "too large" in lib.last_error()
        assert np.all(np.asarray(Cb) == 7.0)
        # pageable matrices are refused as well (the runtime would stage them through buffers of its own)
        P = np.ones((256, 256), order="F")
        rc = lib.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 256, 256, 256, 1.0, P, 256, P, 256, 0.0, P, 256, check=False)
        assert rc == 6
        # argument errors and quick returns are those of blasx_dgemm
        assert lib.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, 5, 8, 8, 8, 1.0, Ab, n, Ab, n, 0.0, Cb, n, check=False) == -3
        assert lib.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 0, 8, 8, 1.0, Ab, n, Ab, n, 0.0, Cb, n, check=False) == 0
    finally:
        lib.set_tile(1024)
        lib.shutdown()
