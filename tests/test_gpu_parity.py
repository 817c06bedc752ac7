"""GPU parity: the HIP path through the C ABI against the CPU oracle, same seeded inputs.

Small and ragged cases compare every element; the benchmark-sized cases compare whole output
tiles (every element of them, the first and the last task of the call among them) and sampled
elements of 64 sampled output tiles (the oracle computes each from the rows of A and columns of B
it needs).  Two gates on every comparison:
  normwise    ||got - want||_F / ||want||_F  <  1e-13 (fp64), 1e-5 (fp32); TRSM also by the
              residual ||op(A) X - alpha B|| / (||A|| ||X||) <= 1e-13;
  elementwise |got - want|_ij <= 8 u |alpha| ||row i of op(A)||_2 ||column j of op(B)||_2
              + 4 u |beta C_ij|  (+ one rounding of the result in single precision),
              u = 2^-53 or 2^-24.  For the zero-mean random operands used here the error of a
              length-K sum, in whatever order, has a standard deviation below 0.6 u ||a|| ||b||
              (each addition errs by at most u/2 of a partial sum whose own spread is
              sqrt(k) sigma_a sigma_b), so the bound is beyond ten deviations whatever K is,
              while one wrong element with a relative error of 1e-10 fails it.  It is always
              below the worst-case bound K u (|A||B|)_ij once K > 16.  The one place where the terms
              of a sum are not zero-mean -- the diagonal of A A^T, a sum of squares -- gets the
              worst-case bound instead (square_sums).
Integer-valued inputs make every product and sum exact: those cases must match bit for bit, so
that a mistake at a tile, macro-tile or chain boundary shows as a mismatch and not as a small error.
"""
import itertools

import numpy as np
import pytest

import oracle as ref
import synth
from paper_1510_05041_amd import blasx

pytestmark = pytest.mark.gpu

# the mutant tests of the oracle's pins swap its library through the environment: never here
assert not ref.overridden(), "ORACLE_LIB_OVERRIDE must not be set when the GPU path is judged"

TOL64, TOL32 = 1e-13, 1e-5
U64, U32 = 2.0 ** -53, 2.0 ** -24
TRANS = [blasx.NoTrans, blasx.Trans]


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available()
    L = blasx.default()
    yield L
    L.shutdown()


def configure(L, T, nstreams=4, arena_gb=2.0, cap_bytes=0, **opts):
    L.init(int(arena_gb * 2 ** 30), nstreams=nstreams)
    L.set_tile(T)
    L.set_cache_bytes(cap_bytes)
    defaults = dict(group=16, kchain=4, depth=6, rs=32, sb_rows=4, sb_cols=4, shells=1, priority=1, profile=0, persist=0, wide=0, ramp=0,
                    merge=0, late_c=1, row_order=1, tail_cut=4, stagger_panels=2, stagger_lag=0)
    defaults.update(opts)
    for k, v in defaults.items():
        L.set_option(k, v)
    L.reset_stats()


def pinned(rows, cols, seed, mat, dtype=np.float64, ld=None, integers=False):
    a, owner = blasx.pinned_matrix(rows, cols, dtype=dtype, ld=ld)
    if rows and cols:
        synth.fill(a, seed, mat, integers=integers)
    return a, owner


def relerr(got, want):
    want = np.asarray(want, dtype=np.float64)
    return np.linalg.norm(np.asarray(got, dtype=np.float64) - want) / max(np.linalg.norm(want), 1e-300)


def norms(x, axis):
    """2-norms of the rows (axis=1) or columns (axis=0) of x in double precision; NaN counts as zero
    (poisoned entries are never operands)."""
    x = np.nan_to_num(np.asarray(x, dtype=np.float64))
    return np.sqrt(np.einsum("ij,ij->i" if axis == 1 else "ij,ij->j", x, x))


def elem_bound(row_norms, col_norms, alpha=1.0, beta_c=None, single=False, want=None, c=8.0):
    """The elementwise bound of the module docstring as a matrix."""
    u = U32 if single else U64
    b = c * u * abs(alpha) * np.outer(row_norms, col_norms)
    if beta_c is not None:
        b = b + 4 * u * np.abs(np.asarray(beta_c, dtype=np.float64))
    if single and want is not None:
        b = b + u * np.abs(np.asarray(want, dtype=np.float64))
    return b + 1e-300


def square_sums(row_norms, K, alpha=1.0, single=False, gi=None, gj=None):
    """Extra allowance where an output element is a sum of squares (the diagonal of A A^T): the terms are all of one
    sign, the partial sums grow like k instead of sqrt(k), and the bound of zero-mean data does not apply; there the
    worst-case bound 2 K u sum(a^2) (K u for the oracle's sum, K u for the kernel's) is taken.  gi, gj: global row and
    column indices of the compared block (default: a whole square matrix)."""
    n = len(row_norms)
    gi = np.arange(n) if gi is None else np.asarray(gi)
    gj = np.arange(n) if gj is None else np.asarray(gj)
    u = U32 if single else U64
    same = gi[:, None] == gj[None, :]
    return same * (2.0 * K * u * abs(alpha) * np.asarray(row_norms)[:, None] ** 2)


def assert_close(got, want, bound, tol, what="", mask=None):
    """Both gates: normwise relative error below tol and every element within its bound."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if mask is not None:
        got, want, bound = got[mask], want[mask], np.broadcast_to(bound, mask.shape)[mask]
    assert np.all(np.isfinite(got)), what
    err = relerr(got, want)
    assert err < tol, (what, err)
    ratio = np.abs(got - want) / bound
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= 1.0, (what, "elementwise bound exceeded by x%.3g at %d elements" % (worst, int((ratio > 1).sum())))
    return err


def op(x, trans):
    return np.asarray(x) if trans == blasx.NoTrans else np.asarray(x).T


def tri_matrix(A, uplo, diag):
    """The triangular matrix that (A, uplo, diag) stands for, in double precision."""
    a = np.nan_to_num(np.asarray(A, dtype=np.float64))
    t = np.tril(a) if uplo == blasx.Lower else np.triu(a)
    if diag == blasx.Unit:
        np.fill_diagonal(t, 1.0)
    return t


def trmm_bound(side, uplo, trans, diag, A, B0, alpha, single=False, want=None, c=8.0):
    """Elementwise bound for B <- alpha op(T) B0 (left) or alpha B0 op(T) (right)."""
    t = op(tri_matrix(A, uplo, diag), trans)
    if side == blasx.Left:
        return elem_bound(norms(t, 1), norms(B0, 0), alpha, single=single, want=want, c=c)
    return elem_bound(norms(B0, 1), norms(t, 0), alpha, single=single, want=want, c=c)


def assert_trsm_residual(side, uplo, trans, diag, A, X, B0, alpha, tol, what="", single=False):
    """||op(T) X - alpha B0|| / (||T|| ||X||) < tol, the product formed by the oracle's TRMM, and the same
    residual element by element against 16 u ||row of op(T)|| ||column of X|| (+ 4 u |alpha B0|): the
    solve multiplies by explicitly inverted diagonal tiles, whose residual carries the (small, the
    triangles are diagonally dominant) condition number of a diagonal tile."""
    X = np.array(X, order="F")
    assert np.all(np.isfinite(X)), what
    R = X.copy(order="F")
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 1.0, np.asarray(A), R)
    t = tri_matrix(A, uplo, diag)
    res = np.linalg.norm(R.astype(np.float64) - alpha * np.asarray(B0, dtype=np.float64)) / (np.linalg.norm(t) * np.linalg.norm(X.astype(np.float64)))
    assert res < tol, (what, res)
    bound = trmm_bound(side, uplo, trans, diag, A, X, 1.0, single=single, want=R if single else None, c=16.0)
    bound = bound + 4 * (U32 if single else U64) * np.abs(alpha * np.asarray(B0, dtype=np.float64))
    ratio = np.abs(R.astype(np.float64) - alpha * np.asarray(B0, dtype=np.float64)) / bound
    assert ratio.max() <= 1.0, (what, "elementwise residual bound exceeded by x%.3g" % ratio.max())
    return res


def sym_matrix(A, uplo):
    a = np.nan_to_num(np.asarray(A, dtype=np.float64))
    t = np.tril(a) if uplo == blasx.Lower else np.triu(a)
    return t + t.T - np.diag(np.diag(t))


# ------------------------------------------------------------------ small, full compare --

def test_config1_dgemm_1024_tile256_two_streams_full_output(lib):
    """DGEMM NN, M=N=K=1024, uniform[-1,1] seed 0, alpha=1, beta=0.5, T=256, 2 streams."""
    n = 1024
    configure(lib, T=256, nstreams=2, arena_gb=0.25)
    A, ka = pinned(n, n, 0, synth.MAT_A)
    B, kb = pinned(n, n, 0, synth.MAT_B)
    C, kc = pinned(n, n, 0, synth.MAT_C)
    C0 = np.array(C, order="F")
    want = np.array(C, order="F")
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.5, C, n)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.asarray(A), np.asarray(B), 0.5, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(B, 0), 1.0, 0.5 * C0), TOL64)
    st = lib.get_stats()
    assert st["tasks"] == 16 and st["tile_steps"] == 64
    assert st["bytes_h2d"] == 3 * 8 * n * n and st["bytes_d2h"] == 8 * n * n


def test_arena_and_streams_of_the_library_itself_across_inits(lib):
    """blasx_init with no arena and no streams: the library allocates both; a later init with a smaller
    or equal arena uses the kept one again, a larger one replaces it, blasx_shutdown frees it."""
    n = 640
    A, ka = pinned(n, n, 3, synth.MAT_A)
    B, kb = pinned(n, n, 3, synth.MAT_B)
    C, kc = pinned(n, n, 3, synth.MAT_C)
    C0 = np.array(C, order="F")
    want = np.array(C0, order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.asarray(A), np.asarray(B), -1.0, want)
    for step, mib in enumerate((256, 128, 256, 512, 64)):
        if step == 4:
            lib.shutdown()
        lib.init_raw(mib * 2 ** 20, 0)
        lib.set_tile(128)
        lib.set_cache_bytes(0)
        for k, v in dict(group=4, kchain=4, depth=6, rs=32, profile=0, persist=0, wide=0, ramp=0).items():
            lib.set_option(k, v)
        C[...] = C0
        lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, -1.0, C, n)
        assert_close(C, want, elem_bound(norms(A, 1), norms(B, 0), 1.0, C0), TOL64, (step, mib))
    lib.shutdown()


@pytest.mark.parametrize("order", [blasx.ColMajor, blasx.RowMajor])
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_dgemm_ragged_all_transposes(lib, order, ta, tb):
    """Several tiles, ragged tails in every dimension, padded leading dimensions."""
    M, N, K = 389, 270, 333
    configure(lib, T=128, arena_gb=0.25, group=5, kchain=3)
    rng = np.random.default_rng(M + ta + 2 * tb + order)
    shape_a = (M, K) if ta == blasx.NoTrans else (K, M)
    shape_b = (K, N) if tb == blasx.NoTrans else (N, K)

    def stored(shape, pad):
        """(logical view, array whose address is passed, leading dimension, owner)."""
        r, c = shape
        if order == blasx.ColMajor:
            v, owner = blasx.pinned_matrix(r, c, ld=r + pad)
            logical = v
        else:   # a row-major r x c matrix is the column-major c x r matrix of its transpose
            v, owner = blasx.pinned_matrix(c, r, ld=c + pad)
            logical = v.T
        logical[...] = rng.uniform(-1, 1, (r, c))
        return logical, v, v.strides[1] // 8, owner

    A, pa, lda, ka = stored(shape_a, 3)
    B, pb, ldb, kb = stored(shape_b, 0)
    C, pc, ldc, kc = stored((M, N), 5)
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.dgemm(order, ta, tb, M, N, K, -0.75, pa, lda, pb, ldb, 0.3, pc, ldc)
    opa = np.asarray(A) if ta == blasx.NoTrans else np.asarray(A).T
    opb = np.asarray(B) if tb == blasx.NoTrans else np.asarray(B).T
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, -0.75, np.asfortranarray(opa), np.asfortranarray(opb), 0.3, want)
    assert_close(C, want, elem_bound(norms(opa, 1), norms(opb, 0), -0.75, 0.3 * C0), TOL64)


def test_dgemm_integer_inputs_bit_exact(lib):
    M, N, K = 640, 384, 1000
    configure(lib, T=256, arena_gb=0.25)
    A, ka = pinned(M, K, 3, 0, integers=True)
    B, kb = pinned(K, N, 3, 1, integers=True)
    C, kc = pinned(M, N, 3, 2, integers=True)
    want = 2.0 * (np.asarray(A) @ np.asarray(B)) - np.asarray(C)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 2.0, A, M, B, K, -1.0, C, M)
    assert np.array_equal(np.asarray(C), want)


def test_dgemm_beta_zero_ignores_nan_and_empty_inputs(lib):
    M, N, K = 300, 200, 260
    configure(lib, T=128, arena_gb=0.25)
    A, ka = pinned(M, K, 4, 0)
    B, kb = pinned(K, N, 4, 1)
    C, kc = blasx.pinned_matrix(M, N)
    C[...] = np.nan
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 1.0, A, M, B, K, 0.0, C, M)
    want = np.zeros((M, N), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.asarray(A), np.asarray(B), 0.0, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(B, 0)), TOL64)
    before = np.array(C)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 0, N, K, 1.0, A, M, B, K, 0.0, C, M)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, 0, 1.0, A, M, B, 1, 1.0, C, M)
    assert np.array_equal(np.asarray(C), before)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, 0, 1.0, A, M, B, 1, 2.0, C, M)
    assert np.array_equal(np.asarray(C), 2.0 * before)


def test_dgemm_pageable_host_memory(lib):
    """Plain numpy (not page-locked) matrices still work, only without asynchronous DMA."""
    n = 512
    configure(lib, T=128, arena_gb=0.25)
    A, B, C = synth.matrix(n, n, 5, 0), synth.matrix(n, n, 5, 1), synth.matrix(n, n, 5, 2)
    want = C.copy(order="F")
    C0 = C.copy(order="F")
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, A, B, 1.0, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(B, 1), 1.0, C0), TOL64)


def test_sgemm_small_full_compare(lib):
    M, N, K = 700, 520, 900
    configure(lib, T=256, arena_gb=0.25)
    A, ka = pinned(M, K, 6, 0, dtype=np.float32)
    B, kb = pinned(N, K, 6, 1, dtype=np.float32)
    C, kc = pinned(M, N, 6, 2, dtype=np.float32)
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.sgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, M, N, K, 1.0, A, M, B, N, 1.0, C, M)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, np.asarray(A), np.asarray(B), 1.0, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(B, 1), 1.0, C0, single=True, want=want), TOL32)


def test_dgemm_capped_cache_eviction(lib):
    """Tile cache capped to 40 slots while A and B have 128 tiles: ALRU must evict and refetch."""
    n, T = 2048, 256
    configure(lib, T=T, arena_gb=0.25, cap_bytes=40 * T * T * 8, group=8, kchain=2)
    A, ka = pinned(n, n, 7, 0)
    B, kb = pinned(n, n, 7, 1)
    C, kc = pinned(n, n, 7, 2)
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.asarray(A), np.asarray(B), 1.0, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(B, 0), 1.0, C0), TOL64)
    st = lib.get_stats()
    assert st["peak_slots"] <= 40 and st["evictions"] > 0 and st["refetches"] > 0
    assert st["misses"] == 128 + st["refetches"]


def test_run_to_run_bit_reproducible(lib):
    n = 1536
    configure(lib, T=256, arena_gb=0.5)
    A, ka = pinned(n, n, 8, 0)
    B, kb = pinned(n, n, 8, 1)
    outs = []
    for _ in range(3):
        C, kc = blasx.pinned_matrix(n, n)
        C[...] = 0
        lib.dgemm(blasx.ColMajor, blasx.Trans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
        outs.append(np.array(C))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ------------------------------------------------------------------ SYRK / TRMM / TRSM ---

@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_dsyrk_small_full_compare(lib, uplo, trans):
    N, K = 650, 410
    configure(lib, T=128, arena_gb=0.25, group=6)
    A, ka = pinned(*((N, K) if trans == blasx.NoTrans else (K, N)), 9, 0)
    C, kc = pinned(N, N, 9, 2)
    other = np.triu_indices(N, 1) if uplo == blasx.Lower else np.tril_indices(N, -1)
    C[other] = 4321.5
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.dsyrk(blasx.ColMajor, uplo, trans, N, K, 0.9, A, A.shape[0], 1.0, C, N)
    ref.syrk(ref.ColMajor, uplo, trans, 0.9, np.asarray(A), 1.0, want)
    assert np.all(np.asarray(C)[other] == 4321.5)
    rn = norms(op(A, trans), 1)
    assert_close(C, want, elem_bound(rn, rn, 0.9, C0) + square_sums(rn, K, 0.9), TOL64)


@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_dsyr2k_small_full_compare(lib, uplo, trans):
    N, K = 650, 410
    configure(lib, T=128, arena_gb=0.25, group=6)
    shape = (N, K) if trans == blasx.NoTrans else (K, N)
    A, ka = pinned(*shape, 14, 0)
    B, kb = pinned(*shape, 14, 1)
    C, kc = pinned(N, N, 14, 2)
    other = np.triu_indices(N, 1) if uplo == blasx.Lower else np.tril_indices(N, -1)
    C[other] = -8765.25
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.dsyr2k(blasx.ColMajor, uplo, trans, N, K, 0.6, A, A.shape[0], B, B.shape[0], -1.0, C, N)
    ref.syr2k(ref.ColMajor, uplo, trans, 0.6, np.asarray(A), np.asarray(B), -1.0, want)
    assert np.all(np.asarray(C)[other] == -8765.25)
    ra, rb = norms(op(A, trans), 1), norms(op(B, trans), 1)
    assert_close(C, want, elem_bound(ra, rb, 0.6, C0) + elem_bound(rb, ra, 0.6), TOL64)


@pytest.mark.parametrize("order", [blasx.ColMajor, blasx.RowMajor])
@pytest.mark.parametrize("side", [blasx.Left, blasx.Right])
@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
def test_dsymm_small_full_compare(lib, order, side, uplo):
    M, N = 530, 390
    configure(lib, T=128, arena_gb=0.25, group=6)
    na = M if side == blasx.Left else N
    A, ka = pinned(na, na, 15, 0)
    # the triangle that is not stored, in terms of the logical matrix
    logical_other = np.triu_indices(na, 1) if uplo == blasx.Lower else np.tril_indices(na, -1)
    r, c = (M, N) if order == blasx.ColMajor else (N, M)   # array extents as column-major storage
    B, kb = pinned(r, c, 15, 1)
    C, kc = pinned(r, c, 15, 2)
    if order == blasx.ColMajor:
        A[logical_other] = np.nan
        Ar, Br, want = np.asarray(A), np.asarray(B), np.array(C, order="F")
    else:
        A[logical_other[1], logical_other[0]] = np.nan     # the column-major array is the transpose
        Ar, Br, want = np.asarray(A).T, np.asarray(B).T, np.array(np.asarray(C).T, order="C")
    C0 = np.array(want)
    lib.dsymm(order, side, uplo, M, N, 1.3, A, na, B, r, 0.5, C, r)
    ref.symm(order, side, uplo, 1.3, Ar, Br, 0.5, want)
    got = np.asarray(C) if order == blasx.ColMajor else np.asarray(C).T
    S = sym_matrix(Ar, uplo)
    bound = elem_bound(norms(S, 1), norms(Br, 0), 1.3, 0.5 * C0) if side == blasx.Left else elem_bound(norms(Br, 1), norms(S, 0), 1.3, 0.5 * C0)
    assert_close(got, want, bound, TOL64)


FLAGS = list(itertools.product([blasx.Left, blasx.Right], [blasx.Upper, blasx.Lower], TRANS, [blasx.NonUnit, blasx.Unit]))


def triangular(n, seed, uplo, diag):
    A, ka = pinned(n, n, seed, 0)
    synth.dominant_diag(A, seed, 0)
    if diag == blasx.Unit:
        A[...] = np.asarray(A) / n
    outside = np.triu_indices(n, 1) if uplo == blasx.Lower else np.tril_indices(n, -1)
    A[outside] = np.nan                      # never read
    if diag == blasx.Unit:
        A[np.diag_indices(n)] = np.nan       # never read either
    return A, ka


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_dtrmm_small_full_compare(lib, side, uplo, trans, diag):
    M, N = 530, 390
    configure(lib, T=128, arena_gb=0.25, group=6)
    A, ka = triangular(M if side == blasx.Left else N, 10, uplo, diag)
    B, kb = pinned(M, N, 10, 1)
    want = np.array(B, order="F")
    B0 = np.array(B, order="F")
    lib.dtrmm(blasx.ColMajor, side, uplo, trans, diag, M, N, 1.1, A, A.shape[0], B, M)
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 1.1, np.asarray(A), want)
    assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, 1.1), TOL64)


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_dtrsm_small_full_compare_and_residual(lib, side, uplo, trans, diag):
    M, N = 530, 390
    configure(lib, T=128, arena_gb=0.25, group=6)
    n = M if side == blasx.Left else N
    A, ka = triangular(n, 11, uplo, diag)
    B, kb = pinned(M, N, 11, 1)
    B0 = np.array(B, order="F")
    want = np.array(B, order="F")
    lib.dtrsm(blasx.ColMajor, side, uplo, trans, diag, M, N, 0.7, A, n, B, M)
    ref.trsm(ref.ColMajor, side, uplo, trans, diag, 0.7, np.asarray(A), want)
    X = np.array(B, order="F")
    assert np.all(np.isfinite(X))
    assert relerr(X, want) < TOL64
    assert_trsm_residual(side, uplo, trans, diag, A, X, B0, 0.7, TOL64)


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_dtrmm_dtrsm_tiles_of_several_macro_tiles(lib, side, uplo, trans, diag):
    """Tile-aligned 1024 x 1024 with T = 512: a triangular tile spans 4 x 4 macro-tiles, so the kernel
    that masks triangular operands skips the slabs outside the triangle (a different k range per
    macro-tile), masks only the slabs that cross the diagonal, and hands its macro-tiles out longest
    first.  NaN outside the stored triangle must never be read."""
    M = N = 1024
    configure(lib, T=512, arena_gb=0.25, group=4)
    A, ka = triangular(M, 41, uplo, diag)
    B, kb = pinned(M, N, 41, 1)
    B0 = np.array(B, order="F")
    want = np.array(B, order="F")
    lib.dtrmm(blasx.ColMajor, side, uplo, trans, diag, M, N, 0.8, A, M, B, M)
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 0.8, np.asarray(A), want)
    assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, 0.8), TOL64)
    B[...] = B0
    lib.dtrsm(blasx.ColMajor, side, uplo, trans, diag, M, N, 0.8, A, M, B, M)
    assert_trsm_residual(side, uplo, trans, diag, A, B, B0, 0.8, TOL64)


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS[::5])
def test_strmm_tiles_of_several_macro_tiles(lib, side, uplo, trans, diag):
    """Same in single precision (slabs are 32 deep there)."""
    M = N = 1024
    configure(lib, T=512, arena_gb=0.25, group=4)
    A64, ka = triangular(M, 42, uplo, diag)
    A, k32 = blasx.pinned_matrix(M, M, dtype=np.float32)
    A[...] = np.asarray(A64).astype(np.float32)
    B, kb = pinned(M, N, 42, 1, dtype=np.float32)
    want = np.array(B, order="F")
    B0 = np.array(B, order="F")
    lib.strmm(blasx.ColMajor, side, uplo, trans, diag, M, N, 1.2, A, M, B, M)
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 1.2, np.asarray(A), want)
    assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, 1.2, single=True, want=want), TOL32)


# ------------------------------------------------------------------ benchmark sizes, sampled --

def sampled_positions(T, rows, cols, rng, count=8):
    """Tile-local row and column positions: edges of the tile and of the 128-wide macro-tiles, plus random ones."""
    def pick(extent):
        fixed = [p for p in (0, 127, 128, extent - 1) if 0 <= p < extent]
        rand = rng.integers(0, extent, size=max(0, count - len(fixed))).tolist()
        return sorted(set(fixed + rand))
    return pick(rows), pick(cols)


def check_gemm_sampled(ta, tb, M, N, K, alpha, A, B, beta, C_before_fn, C, T, seed, tol, dtype=np.float64):
    """Oracle on sampled elements of 64 sampled output tiles, both gates; returns the worst tile error."""
    rng = np.random.default_rng(seed)
    ntm, ntn = -(-M // T), -(-N // T)
    single = np.dtype(dtype) == np.float32
    worst = 0.0
    for (ti, tj) in synth.sample_tiles(ntm, ntn, 64, seed):
        rows, cols = sampled_positions(T, min(T, M - ti * T), min(T, N - tj * T), rng)
        gi = np.array(rows) + ti * T
        gj = np.array(cols) + tj * T
        a = np.asarray(A[gi, :] if ta == blasx.NoTrans else A[:, gi].T, dtype=dtype, order="F")
        b = np.asarray(B[:, gj] if tb == blasx.NoTrans else B[gj, :].T, dtype=dtype, order="F")
        c0 = C_before_fn(gi, gj).astype(dtype)
        want = np.asfortranarray(c0)
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, alpha, a, b, beta, want)
        got = np.asarray(C)[np.ix_(gi, gj)]
        bound = elem_bound(norms(a, 1), norms(b, 0), alpha, beta * c0.astype(np.float64), single=single, want=want)
        worst = max(worst, assert_close(got, want, bound, tol, "tile (%d, %d)" % (ti, tj)))
    return worst


def whole_tiles(ntm, ntn, count, seed):
    """Tile indices for whole-tile comparison: the first and the last tile of the matrix (the first and the
    last task of a call in queue order or nearly so), then sampled ones; all of them if count covers them."""
    if count >= ntm * ntn:
        return [(i, j) for i in range(ntm) for j in range(ntn)]
    picked = [(0, 0), (ntm - 1, ntn - 1)]
    for t in synth.sample_tiles(ntm, ntn, ntm * ntn if ntm * ntn < 4 * count else 4 * count, seed + 77):
        if len(picked) >= count:
            break
        if t not in picked:
            picked.append(t)
    return picked[:count]


def check_gemm_whole_tiles(ta, tb, M, N, K, alpha, A, B, beta, c_seed, C, T, count, seed, tol, dtype=np.float64):
    """Oracle on EVERY element of `count` output tiles (block rows of op(A) times block columns of op(B));
    c_seed = (seed, matrix id) of the generator that made C before the call, or None for beta = 0."""
    ntm, ntn = -(-M // T), -(-N // T)
    single = np.dtype(dtype) == np.float32
    worst = 0.0
    for (ti, tj) in whole_tiles(ntm, ntn, count, seed):
        r0, r1, c0, c1 = ti * T, min(M, ti * T + T), tj * T, min(N, tj * T + T)
        # views of the host matrices as they are stored: the oracle takes the transposition flags itself.  (A transposed
        # A is handed over as a transposed copy instead: the oracle's inner loop runs over the rows of op(A), which in the
        # stored transpose are a whole leading dimension apart.)
        ta_ref = ta
        if ta == blasx.NoTrans:
            a = A[r0:r1, :]
        else:
            a, ta_ref = np.asfortranarray(A[:, r0:r1].T), blasx.NoTrans
        b = B[:, c0:c1] if tb == blasx.NoTrans else B[c0:c1, :]
        if c_seed is None:
            before = np.zeros((r1 - r0, c1 - c0), dtype=dtype, order="F")
        else:
            before = synth.block(c_seed[0], c_seed[1], M, r0, c0, r1 - r0, c1 - c0, dtype=dtype)
        want = np.array(before, order="F")
        ref.gemm(ref.ColMajor, ta_ref, tb, alpha, a, b, beta, want)
        got = np.asarray(C)[r0:r1, c0:c1]
        bound = elem_bound(norms(a, 1 if ta_ref == blasx.NoTrans else 0), norms(b, 0 if tb == blasx.NoTrans else 1), alpha,
                           beta * before.astype(np.float64), single=single, want=want)
        worst = max(worst, assert_close(got, want, bound, tol, "whole tile (%d, %d)" % (ti, tj)))
    return worst


@pytest.mark.parametrize("n", [4096, 8192])
def test_config2_dgemm_square_sampled(lib, n):
    """DGEMM NN, alpha=beta=1, T=1024, 4 streams, host-resident; 64 sampled tiles."""
    configure(lib, T=1024, nstreams=4, arena_gb=8.0)
    A, ka = pinned(n, n, 0, synth.MAT_A)
    B, kb = pinned(n, n, 0, synth.MAT_B)
    C, kc = pinned(n, n, 0, synth.MAT_C)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
    before = lambda gi, gj: np.array([[synth.element(0, synth.MAT_C, int(i), int(j), n) for j in gj] for i in gi])
    check_gemm_sampled(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 1.0, before, C, 1024, n, TOL64)
    # every element of every output tile
    check_gemm_whole_tiles(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 1.0, (0, synth.MAT_C), C, 1024, 64, n, TOL64)
    st = lib.get_stats()
    assert st["bytes_h2d"] == 3 * 8 * n * n and st["evictions"] == 0


def report(name, lib, flop, seconds):
    st = lib.get_stats()
    print("\n[result] %s: %.3f s, %.1f TFLOP/s; h2d %.2f GB d2h %.2f GB; hits %d misses %d evictions %d refetches %d "
          "slot_waits %d peak_slots %d launches %d" % (
              name, seconds, flop / seconds / 1e12, st["bytes_h2d"] / 1e9, st["bytes_d2h"] / 1e9, st["hits"], st["misses"],
              st["evictions"], st["refetches"], st["slot_waits"], st["peak_slots"], st["launches"]), flush=True)
    return st


def timed(fn):
    import time
    t0 = time.perf_counter()
    fn()
    return time.perf_counter() - t0


def c_before(seed, mat, rows):
    return lambda gi, gj: np.array([[synth.element(seed, mat, int(i), int(j), rows) for j in gj] for i in gi])


AUTO = dict(group=0, kchain=0, wide=11)      # the library's own choices: what bench.py times


@pytest.mark.parametrize("schedule", ["grouped", "auto"])
@pytest.mark.parametrize("n", [16384, 32768])
def test_config2_dgemm_large_sampled(lib, n, schedule):
    """The benchmark workload itself (N=32768) and the size below it: in the launch configuration bench.py times
    (all tasks advance together, C tiles arrive late) and in the grouped schedule (16 tasks run to completion)."""
    tiles = 512 if schedule == "auto" else 160
    opts = AUTO if schedule == "auto" else {}
    configure(lib, T=1024, nstreams=4, arena_gb=((3 if schedule == "auto" else 2) * 8 * n * n + tiles * 8 * 2 ** 20) / 2 ** 30, **opts)
    A, ka = pinned(n, n, 0, synth.MAT_A)
    B, kb = pinned(n, n, 0, synth.MAT_B)
    C, kc = pinned(n, n, 0, synth.MAT_C)
    dt = timed(lambda: lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n))
    st = report("cfg2 DGEMM NN N=%d T=1024 %s" % (n, schedule), lib, 2.0 * n ** 3, dt)
    check_gemm_sampled(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 1.0, c_before(0, synth.MAT_C, n), C, 1024, n, TOL64)
    check_gemm_whole_tiles(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 1.0, (0, synth.MAT_C), C, 1024, 4, n, TOL64)
    assert st["bytes_h2d"] == 3 * 8 * n * n and st["bytes_d2h"] == 8 * n * n and st["refetches"] == 0
    assert lib.get_option("last_wide") == (1 if schedule == "auto" else 0)
    # one inbound copy per tile counted, and (in the configuration bench.py times) most tiles travelled in company
    assert st["copies_h2d"] == 3 * (n // 1024) ** 2 and st["transfers_h2d"] <= st["copies_h2d"]
    if schedule == "auto":
        assert st["transfers_h2d"] <= 0.4 * st["copies_h2d"], (st["transfers_h2d"], st["copies_h2d"])


@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_wide_schedule_dgemm_ragged_full_compare(lib, ta, tb):
    """The wide schedule on ragged tiles with 17 k-tiles: three rounds of 8, 8 and 1 k-steps, late C tiles."""
    M, N, K = 650, 530, 2100
    configure(lib, T=128, arena_gb=0.5, **AUTO)
    A, ka = pinned(*((M, K) if ta == blasx.NoTrans else (K, M)), 30, 0)
    B, kb = pinned(*((K, N) if tb == blasx.NoTrans else (N, K)), 30, 1)
    C, kc = pinned(M, N, 30, 2)
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.dgemm(blasx.ColMajor, ta, tb, M, N, K, -1.25, A, A.shape[0], B, B.shape[0], 0.75, C, M)
    assert lib.get_option("last_wide") == 1 and lib.get_option("last_kchain") == 8
    ref.gemm(ref.ColMajor, ta, tb, -1.25, np.asarray(A), np.asarray(B), 0.75, want)
    assert_close(C, want, elem_bound(norms(op(A, ta), 1), norms(op(B, tb), 0), -1.25, 0.75 * C0), TOL64)
    st = lib.get_stats()
    assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N) and st["copies_d2h"] == 6 * 5


def poison_arena(lib):
    """Every byte of the tile arena 0xFF: NaN in both precisions wherever the library reads what it has not written."""
    import torch
    lib.arena_tensor().fill_(0xFF)
    torch.cuda.synchronize()


@pytest.mark.parametrize("T", [128, 1024, 208])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_ragged_sizes_run_in_the_fast_kernels_on_zero_padded_tiles(lib, T, dtype):
    """Sizes that are no multiple of anything: tiles are zero-padded in their slots to whole macro-tiles and every
    tile step of the products runs in the unpredicated kernels (the arena starts
    as NaN, so a tile whose padding was not cleared, after its copy or after it was derived on the device, shows).
    With a tile edge that is no multiple of the macro-tile edge (208) the same calls run in the bounds-checked kernel."""
    f64 = dtype == np.float64
    fast = T % 128 == 0
    tol, single = (TOL64, False) if f64 else (TOL32, True)
    gemm, syrk, syr2k, symm, trmm = ((lib.dgemm, lib.dsyrk, lib.dsyr2k, lib.dsymm, lib.dtrmm) if f64 else
                                     (lib.sgemm, lib.ssyrk, lib.ssyr2k, lib.ssymm, lib.strmm))
    M, N, K = (1500, 1300, 2300) if T == 1024 else (650, 530, 1490)
    for wide in (0, 1):
        configure(lib, T=T, arena_gb=1.0, **(dict(group=0, kchain=0, wide=2) if wide else {}))
        poison_arena(lib)
        for ta, tb in itertools.product(TRANS, TRANS):
            A, ka = pinned(*((M, K) if ta == blasx.NoTrans else (K, M)), 70, 0, dtype=dtype)
            B, kb = pinned(*((K, N) if tb == blasx.NoTrans else (N, K)), 70, 1, dtype=dtype)
            C, kc = pinned(M, N, 70, 2, dtype=dtype)
            want, C0 = np.array(C, order="F"), np.array(C, order="F")
            gemm(blasx.ColMajor, ta, tb, M, N, K, -1.25, A, A.shape[0], B, B.shape[0], 0.75, C, M)
            ref.gemm(ref.ColMajor, ta, tb, -1.25, np.asarray(A), np.asarray(B), 0.75, want)
            assert_close(C, want, elem_bound(norms(op(A, ta), 1), norms(op(B, tb), 0), -1.25, 0.75 * C0, single=single, want=want), tol)
        A, ka = pinned(M, K, 71, 0, dtype=dtype)
        B, kb = pinned(M, K, 71, 1, dtype=dtype)
        C, kc = pinned(M, M, 71, 2, dtype=dtype)
        other = np.triu_indices(M, 1)
        C[other] = 1234.5
        want, C0 = np.array(C, order="F"), np.array(C, order="F")
        syrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, M, K, 1.0, A, M, 0.5, C, M)
        ref.syrk(ref.ColMajor, ref.Lower, ref.NoTrans, 1.0, np.asarray(A), 0.5, want)
        ra, rb = norms(A, 1), norms(B, 1)
        assert np.all(np.asarray(C)[other] == 1234.5)
        assert_close(C, want, elem_bound(ra, ra, 1.0, 0.5 * C0, single=single, want=want) + square_sums(ra, K, single=single), tol)
        C1 = np.array(C, order="F")
        want = np.array(C, order="F")
        syr2k(blasx.ColMajor, blasx.Lower, blasx.NoTrans, M, K, 0.5, A, M, B, M, 1.0, C, M)
        ref.syr2k(ref.ColMajor, ref.Lower, ref.NoTrans, 0.5, np.asarray(A), np.asarray(B), 1.0, want)
        assert np.all(np.asarray(C)[other] == 1234.5)
        assert_close(C, want, elem_bound(ra, rb, 0.5, C1, single=single, want=want) + elem_bound(rb, ra, 0.5, single=single), tol)
        for side, uplo in ((blasx.Left, blasx.Lower), (blasx.Right, blasx.Upper)):
            na = M if side == blasx.Left else N
            S, ks = pinned(na, na, 72, 0, dtype=dtype)
            S[np.triu_indices(na, 1) if uplo == blasx.Lower else np.tril_indices(na, -1)] = np.nan
            B, kb = pinned(M, N, 72, 1, dtype=dtype)
            C, kc = pinned(M, N, 72, 2, dtype=dtype)
            want, C0 = np.array(C, order="F"), np.array(C, order="F")
            symm(blasx.ColMajor, side, uplo, M, N, -1.5, S, na, B, M, 0.25, C, M)
            ref.symm(ref.ColMajor, side, uplo, -1.5, np.asarray(S), np.asarray(B), 0.25, want)
            full = sym_matrix(S, uplo)
            bound = (elem_bound(norms(full, 1), norms(B, 0), -1.5, 0.25 * C0, single=single, want=want) if side == blasx.Left
                     else elem_bound(norms(B, 1), norms(full, 0), -1.5, 0.25 * C0, single=single, want=want))
            assert_close(C, want, bound, tol)
        st = lib.get_stats()
        assert st["tile_steps"] > 0 and st["steps_general"] == (0 if fast else st["tile_steps"])
        P, kp = pinned(M, M, 73, 0, dtype=dtype)
        synth.dominant_diag(P, 73, 0)
        P[np.triu_indices(M, 1)] = np.nan
        B, kb = pinned(M, N, 73, 1, dtype=dtype)
        want, B0 = np.array(B, order="F"), np.array(B, order="F")
        trmm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, -0.8, P, M, B, M)
        ref.trmm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, -0.8, np.asarray(P), want)
        assert_close(B, want, trmm_bound(blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, P, B0, -0.8, single=single, want=want), tol)
        st2 = lib.get_stats()
        assert st2["tile_steps"] > st["tile_steps"] and st2["steps_general"] == (0 if fast else st2["tile_steps"])
        # the solve: its results become operands of later steps and are padded when they are adopted
        for side, uplo in ((blasx.Left, blasx.Upper), (blasx.Right, blasx.Lower)):
            na = M if side == blasx.Left else N
            P, kp = pinned(na, na, 74, 0, dtype=dtype)
            synth.dominant_diag(P, 74, 0)
            P[np.tril_indices(na, -1) if uplo == blasx.Upper else np.triu_indices(na, 1)] = np.nan
            B, kb = pinned(M, N, 74, 1, dtype=dtype)
            B0 = np.array(B, order="F")
            trsm = lib.dtrsm if f64 else lib.strsm
            trsm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.NonUnit, M, N, 1.5, P, na, B, M)
            assert_trsm_residual(side, uplo, blasx.NoTrans, blasx.NonUnit, P, B, B0, 1.5, tol, single=not f64)
        st3 = lib.get_stats()
        assert st3["tile_steps"] > st2["tile_steps"] and st3["steps_general"] == (0 if fast else st3["tile_steps"])


def test_wide_schedule_symmetric_routines_full_compare(lib):
    N, K = 650, 1700
    configure(lib, T=128, arena_gb=0.5, **AUTO)
    A, ka = pinned(N, K, 31, 0)
    B, kb = pinned(N, K, 31, 1)
    C, kc = pinned(N, N, 31, 2)
    other = np.triu_indices(N, 1)
    C[other] = 1234.5
    want = np.array(C, order="F")
    lib.dsyrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, N, K, 1.0, A, N, 0.0, C, N)     # beta = 0: diagonal tiles still need C
    assert lib.get_option("last_wide") == 1
    ref.syrk(ref.ColMajor, ref.Lower, ref.NoTrans, 1.0, np.asarray(A), 0.0, want)
    ra, rb = norms(A, 1), norms(B, 1)
    assert np.all(np.asarray(C)[other] == 1234.5)
    assert_close(C, want, elem_bound(ra, ra) + square_sums(ra, K) + 4 * U64 * 1234.5, TOL64)
    C1 = np.array(C, order="F")
    lib.dsyr2k(blasx.ColMajor, blasx.Lower, blasx.NoTrans, N, K, 0.5, A, N, B, N, 1.0, C, N)
    assert lib.get_option("last_wide") == 1
    ref.syr2k(ref.ColMajor, ref.Lower, ref.NoTrans, 0.5, np.asarray(A), np.asarray(B), 1.0, want)
    assert np.all(np.asarray(C)[other] == 1234.5)
    # (want carries the oracle's SYRK result into the second call, C the library's: both errors add)
    assert_close(C, want, elem_bound(ra, rb, 0.5, C1) + elem_bound(rb, ra, 0.5) + elem_bound(ra, ra) + square_sums(ra, K), TOL64)
    M = 1700
    S, ks = pinned(M, M, 32, 0)
    S[np.tril_indices(M, -1)] = np.nan                       # upper triangle stored
    X, kx = pinned(M, 390, 32, 1)
    Y, ky = pinned(M, 390, 32, 2)
    want = np.array(Y, order="F")
    Y0 = np.array(Y, order="F")
    lib.dsymm(blasx.ColMajor, blasx.Left, blasx.Upper, M, 390, 1.0, S, M, X, M, -1.0, Y, M)
    assert lib.get_option("last_wide") == 1
    ref.symm(ref.ColMajor, ref.Left, ref.Upper, 1.0, np.asarray(S), np.asarray(X), -1.0, want)
    assert_close(Y, want, elem_bound(norms(sym_matrix(S, blasx.Upper), 1), norms(X, 0), 1.0, Y0), TOL64)


@pytest.mark.parametrize("choice", ["fixed", "auto"])
def test_config3_out_of_core_dgemm_capped_cache(lib, choice):
    """M=N=K=49152 fp64 (58 GB of operands), beta=0, T=2048, tile cache capped at 8 GB: ALRU eviction and reuse.
    fixed: 16 tasks, chains of 2, 3 launches in flight; auto: the library's own choice of running set and chain under the cap.
    The size is never reduced: without the host memory for it the case is skipped, with the reason."""
    import psutil
    n, T = 49152, 2048
    need, have = 3 * 8 * n * n * 1.1, psutil.virtual_memory().available
    if have < need:
        pytest.skip("N=49152 needs %.0f GB of page-locked host memory, %.0f GB are available" % (need / 1e9, have / 1e9))
    opts = dict(group=16, kchain=2, depth=3) if choice == "fixed" else dict(AUTO)
    configure(lib, T=T, nstreams=4, arena_gb=8.0, cap_bytes=8 * 2 ** 30, **opts)
    A, ka = pinned(n, n, 0, synth.MAT_A)
    B, kb = pinned(n, n, 0, synth.MAT_B)
    C, kc = blasx.pinned_matrix(n, n)
    dt = timed(lambda: lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, C, n))
    st = report("cfg3 out-of-core DGEMM N=%d T=2048 cap 8 GB %s (group %d, chains of %d, wide %d)" % (
        n, choice, lib.get_option("last_group"), lib.get_option("last_kchain"), lib.get_option("last_wide")), lib, 2.0 * n ** 3, dt)
    assert n == 49152 and st["tasks"] == 24 * 24 and st["tile_steps"] == 24 ** 3
    check_gemm_sampled(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 0.0, lambda gi, gj: np.zeros((len(gi), len(gj))),
                       C, T, 3, TOL64)
    if choice == "fixed":       # every element of four whole tiles (412 GFLOP of oracle work each)
        check_gemm_whole_tiles(blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, B, 0.0, None, C, T, 4, 3, TOL64)
    nt = n // T
    assert st["peak_slots"] <= 256
    assert st["evictions"] > 0 and st["refetches"] > 0
    assert st["misses"] == 2 * nt * nt + st["refetches"]
    assert st["bytes_d2h"] == 8 * n * n


def test_config4_dsyrk_lower_notrans_sampled(lib):
    """DSYRK Lower/NoTrans N=16384 K=8192, alpha=1, beta=1 (beta is not stated in the workload list; 1 as in the GEMM sweep)."""
    N, K, T = 16384, 8192, 1024
    configure(lib, T=T, nstreams=4, arena_gb=8.0)
    A, ka = pinned(N, K, 4, synth.MAT_A)
    C, kc = pinned(N, N, 4, synth.MAT_C)
    dt = timed(lambda: lib.dsyrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, N, K, 1.0, A, N, 1.0, C, N))
    report("cfg4 DSYRK L/N N=16384 K=8192", lib, 1.0 * N * (N + 1) * K, dt)
    rng = np.random.default_rng(4)
    nt = N // T
    before = c_before(4, synth.MAT_C, N)
    worst, seen = 0.0, 0
    for (ti, tj) in synth.sample_tiles(nt, nt, 64, 4):
        rows, cols = sampled_positions(T, T, T, rng)
        gi, gj = np.array(rows) + ti * T, np.array(cols) + tj * T
        got = np.asarray(C)[np.ix_(gi, gj)]
        c0 = before(gi, gj)
        if ti < tj:                                    # upper triangle: must be bit-identical
            assert np.array_equal(got, c0)
            continue
        want = np.asfortranarray(c0)
        ai, aj = np.asfortranarray(A[gi, :]), np.asfortranarray(A[gj, :])
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, ai, aj, 1.0, want)
        mask = (gi[:, None] >= gj[None, :])            # inside a diagonal tile only the lower part is written
        assert np.array_equal(got[~mask], c0[~mask])
        bound = elem_bound(norms(ai, 1), norms(aj, 1), 1.0, c0) + square_sums(norms(ai, 1), K, gi=gi, gj=gj)
        worst = max(worst, assert_close(got, want, bound, TOL64, (ti, tj), mask=mask))
        seen += 1
    assert seen > 10 and worst < TOL64, worst
    # every element of four whole tiles of the triangle: a diagonal one, the last one, two below the diagonal
    for (ti, tj) in [(0, 0), (nt - 1, nt - 1), (nt - 1, 0), (nt // 2, nt // 2 - 1)]:
        r0, c0_ = ti * T, tj * T
        before_t = synth.block(4, synth.MAT_C, N, r0, c0_, T, T)
        want = np.array(before_t, order="F")
        ai, aj = np.asfortranarray(A[r0:r0 + T, :]), np.asfortranarray(A[c0_:c0_ + T, :])
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, ai, aj, 1.0, want)
        got = np.asarray(C)[r0:r0 + T, c0_:c0_ + T]
        mask = (np.arange(r0, r0 + T)[:, None] >= np.arange(c0_, c0_ + T)[None, :])
        assert np.array_equal(got[~mask], before_t[~mask])
        bound = elem_bound(norms(ai, 1), norms(aj, 1), 1.0, before_t) + square_sums(norms(ai, 1), K, gi=np.arange(r0, r0 + T), gj=np.arange(c0_, c0_ + T))
        assert_close(got, want, bound, TOL64, ("whole", ti, tj), mask=mask)


def check_trsm_columns(A, B, M, cols, seed, tol):
    """Left/Lower/NoTrans/NonUnit: residual of the columns `cols` of X (each column is an independent solve):
    normwise, and element by element as in assert_trsm_residual.  The right-hand side is regenerated."""
    X = np.asfortranarray(np.asarray(B)[:, cols])
    assert np.all(np.isfinite(X))
    R = X.copy(order="F")
    ref.trmm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, 1.0, np.asarray(A), R)
    B0 = np.empty((M, len(cols)), order="F")
    for q, j in enumerate(cols):
        B0[:, q:q + 1] = synth.block(seed, synth.MAT_B, M, 0, int(j), M, 1)
    row_sq = np.zeros(M)
    for j in range(M):                       # column by column: the matrix is column-major
        row_sq[j:] += np.square(A[j:, j])
    row_norms = np.sqrt(row_sq)
    norm_a = float(np.sqrt(np.sum(row_sq)))
    res = np.linalg.norm(R - B0) / (norm_a * np.linalg.norm(X))
    assert res < tol, res
    bound = elem_bound(row_norms, norms(X, 0), 1.0, B0, c=16.0)
    ratio = np.abs(R - B0) / bound
    assert ratio.max() <= 1.0, "elementwise residual bound exceeded by x%.3g" % ratio.max()
    return res


@pytest.mark.parametrize("schedule", ["grouped", "auto"])
def test_config4_dtrsm_left_lower_notrans_nonunit_residual(lib, schedule):
    """DTRSM Left/Lower/NoTrans/NonUnit M=N=16384, A with diag = N + uniform[0,1], alpha=1; residual on sampled columns.
    grouped: tasks queued by dependency level, 16 at a time; auto: the wide (right-looking) schedule."""
    M = N = 16384
    T = 1024
    configure(lib, T=T, nstreams=4, arena_gb=12.0, **(AUTO if schedule == "auto" else {}))
    A, ka = pinned(M, M, 5, synth.MAT_A)
    synth.dominant_diag(A, 5, synth.MAT_A)
    B, kb = pinned(M, N, 5, synth.MAT_B)
    dt = timed(lambda: lib.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, 1.0, A, M, B, M))
    report("cfg4 DTRSM L/L/N/N M=N=16384 %s" % schedule, lib, 1.0 * M * M * N, dt)
    assert lib.get_option("last_wide") == (1 if schedule == "auto" else 0)
    # every row of 160 columns of X: 64 of the first block column, 64 of the last (two macro-tile columns each), 16 across a
    # tile boundary in between and 16 single ones (the oracle's triangular product costs M^2 per column)
    rng = np.random.default_rng(5)
    cols = np.unique(np.concatenate([np.arange(96, 160), np.arange(N - 64, N), np.arange(7 * T - 8, 7 * T + 8), rng.choice(N, 16, replace=False)]))
    check_trsm_columns(A, B, M, cols, 5, TOL64)


def test_dtrmm_left_lower_16384_sampled_columns(lib):
    """DTRMM Left/Lower/NoTrans/NonUnit M=N=16384 in place, the library's own choices: wide schedule, tasks sorted by
    length, right-hand sides in two staggered panels (the call is bound by the device).  Whole columns of the result
    against the oracle: both panels, both ends of each, columns across tile boundaries and single ones."""
    M = N = 16384
    T = 1024
    configure(lib, T=0, nstreams=4, arena_gb=12.0, **AUTO)
    A, ka = pinned(M, M, 8, synth.MAT_A)
    iu = np.triu_indices(T, 1)
    for c in range(0, M, T):                             # the strictly upper triangle is never read
        A[:c, c:c + T] = np.nan
        A[c:c + T, c:c + T][iu] = np.nan
    B, kb = pinned(M, N, 8, synth.MAT_B)
    rng = np.random.default_rng(8)
    cols = np.unique(np.concatenate([np.arange(0, 24), np.arange(N // 2 - 12, N // 2 + 12), np.arange(N - 24, N),
                                     np.arange(5 * T - 8, 5 * T + 8), np.arange(11 * T - 8, 11 * T + 8), rng.choice(N, 24, replace=False)]))
    B0 = np.array(np.asarray(B)[:, cols], order="F")
    dt = timed(lambda: lib.dtrmm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, -0.75, A, M, B, M))
    report("DTRMM L/L/N/N M=N=16384 auto", lib, 1.0 * M * M * N, dt)
    assert lib.get_option("last_tile") == T and lib.get_option("last_wide") == 1
    st = lib.get_stats()
    assert st["tasks"] == 256 and st["bytes_d2h"] == 8 * M * N and st["steps_general"] == 0
    assert st["bytes_h2d"] == 8 * (M * N + T * T * 136)      # every tile of B and of the stored triangle once
    want = B0.copy(order="F")
    ref.trmm(ref.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, -0.75, np.asarray(A), want)
    got = np.asarray(B)[:, cols]
    assert_close(got, want, trmm_bound(blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, A, B0, -0.75), TOL64, "dtrmm 16384 columns")


def test_dtrsm_order_20480_takes_2048_tiles_residual(lib):
    """A triangular matrix of order 20480: the automatic tile is 2048 (10 x 2 tiles, wide right-looking solve);
    residual on sampled columns."""
    M, N = 20480, 4096
    configure(lib, T=0, nstreams=4, arena_gb=16.0, **AUTO)
    A, ka = pinned(M, M, 6, synth.MAT_A)
    synth.dominant_diag(A, 6, synth.MAT_A)
    B, kb = pinned(M, N, 6, synth.MAT_B)
    lib.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, 1.0, A, M, B, M)
    assert lib.get_option("last_tile") == 2048 and lib.get_option("last_wide") == 1
    rng = np.random.default_rng(6)
    cols = np.unique(np.concatenate([np.arange(120, 136), np.arange(N - 16, N), rng.choice(N, 8, replace=False)]))
    check_trsm_columns(A, B, M, cols, 6, TOL64)


def test_config5a_dgemm_trans_notrans_long_k_sampled(lib):
    """DGEMM Trans/NoTrans M=N=8192 K=65536 (A stored 65536 x 8192), alpha=beta=1, T=1024."""
    M = N = 8192
    K, T = 65536, 1024
    configure(lib, T=T, nstreams=4, arena_gb=12.0, **AUTO)        # 64 tasks x 64 k-steps: the wide schedule
    A, ka = pinned(K, M, 6, synth.MAT_A)
    B, kb = pinned(K, N, 6, synth.MAT_B)
    C, kc = pinned(M, N, 6, synth.MAT_C)
    dt = timed(lambda: lib.dgemm(blasx.ColMajor, blasx.Trans, blasx.NoTrans, M, N, K, 1.0, A, K, B, K, 1.0, C, M))
    report("cfg5a DGEMM TN 8192x8192x65536", lib, 2.0 * M * N * K, dt)
    check_gemm_sampled(blasx.Trans, blasx.NoTrans, M, N, K, 1.0, A, B, 1.0, c_before(6, synth.MAT_C, M), C, T, 6, TOL64)
    check_gemm_whole_tiles(blasx.Trans, blasx.NoTrans, M, N, K, 1.0, A, B, 1.0, (6, synth.MAT_C), C, T, 8, 6, TOL64)


def test_config5b_sgemm_notrans_trans_sampled(lib):
    """SGEMM NoTrans/Trans M=N=K=32768 fp32, alpha=beta=1, T=2048."""
    n, T = 32768, 2048
    configure(lib, T=T, nstreams=4, arena_gb=(4 * 4 * n * n + 128 * 4 * T * T) / 2 ** 30, **AUTO)
    A, ka = pinned(n, n, 7, synth.MAT_A, dtype=np.float32)
    B, kb = pinned(n, n, 7, synth.MAT_B, dtype=np.float32)
    C, kc = pinned(n, n, 7, synth.MAT_C, dtype=np.float32)
    dt = timed(lambda: lib.sgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, n, B, n, 1.0, C, n))
    report("cfg5b SGEMM NT N=32768 T=2048", lib, 2.0 * n ** 3, dt)
    before = lambda gi, gj: np.array([[np.float32(synth.element(7, synth.MAT_C, int(i), int(j), n)) for j in gj] for i in gi],
                                     dtype=np.float32)
    check_gemm_sampled(blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, B, 1.0, before, C, T, 7, TOL32, dtype=np.float32)
    check_gemm_whole_tiles(blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, B, 1.0, (7, synth.MAT_C), C, T, 4, 7, TOL32, dtype=np.float32)

def test_dsyr2k_lower_notrans_16384_sampled(lib):
    """DSYR2K Lower/NoTrans N=16384 K=8192, alpha=1, beta=1 at the SYRK workload's shape."""
    N, K, T = 16384, 8192, 1024
    configure(lib, T=T, nstreams=4, arena_gb=8.0, **AUTO)
    A, ka = pinned(N, K, 16, synth.MAT_A)
    B, kb = pinned(N, K, 16, synth.MAT_B)
    C, kc = pinned(N, N, 16, synth.MAT_C)
    dt = timed(lambda: lib.dsyr2k(blasx.ColMajor, blasx.Lower, blasx.NoTrans, N, K, 1.0, A, N, B, N, 1.0, C, N))
    st = report("DSYR2K L/N N=16384 K=8192", lib, 2.0 * N * (N + 1) * K, dt)
    nt = N // T
    assert st["tasks"] == nt * (nt + 1) // 2 and st["bytes_d2h"] == 8 * T * T * st["tasks"]
    rng = np.random.default_rng(16)
    before = c_before(16, synth.MAT_C, N)
    worst, seen = 0.0, 0
    for (ti, tj) in synth.sample_tiles(nt, nt, 48, 16):
        rows, cols = sampled_positions(T, T, T, rng)
        gi, gj = np.array(rows) + ti * T, np.array(cols) + tj * T
        got = np.asarray(C)[np.ix_(gi, gj)]
        c0 = before(gi, gj)
        if ti < tj:                                    # upper triangle: must be bit-identical
            assert np.array_equal(got, c0)
            continue
        want = np.asfortranarray(c0)
        ai, aj, bi, bj = (np.asfortranarray(X[g, :]) for X, g in ((A, gi), (A, gj), (B, gi), (B, gj)))
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, ai, bj, 1.0, want)
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, bi, aj, 1.0, want)
        mask = (gi[:, None] >= gj[None, :])
        assert np.array_equal(got[~mask], c0[~mask])
        bound = elem_bound(norms(ai, 1), norms(bj, 1), 1.0, c0) + elem_bound(norms(bi, 1), norms(aj, 1))
        worst = max(worst, assert_close(got, want, bound, TOL64, (ti, tj), mask=mask))
        seen += 1
    assert seen > 10 and worst < TOL64, worst
    # every element of four whole tiles of the triangle
    for (ti, tj) in [(0, 0), (nt - 1, nt - 1), (nt - 1, 0), (nt // 2, nt // 2 - 1)]:
        r0, c0_ = ti * T, tj * T
        before_t = synth.block(16, synth.MAT_C, N, r0, c0_, T, T)
        want = np.array(before_t, order="F")
        ai, aj, bi, bj = A[r0:r0 + T, :], A[c0_:c0_ + T, :], B[r0:r0 + T, :], B[c0_:c0_ + T, :]
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, ai, bj, 1.0, want)
        ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, bi, aj, 1.0, want)
        got = np.asarray(C)[r0:r0 + T, c0_:c0_ + T]
        mask = (np.arange(r0, r0 + T)[:, None] >= np.arange(c0_, c0_ + T)[None, :])
        assert np.array_equal(got[~mask], before_t[~mask])
        bound = elem_bound(norms(ai, 1), norms(bj, 1), 1.0, before_t) + elem_bound(norms(bi, 1), norms(aj, 1))
        assert_close(got, want, bound, TOL64, ("whole", ti, tj), mask=mask)


@pytest.mark.parametrize("side,uplo", [(blasx.Left, blasx.Lower), (blasx.Right, blasx.Upper)])
def test_dsymm_16384_sampled(lib, side, uplo):
    """DSYMM M=N=16384, alpha=1, beta=1; the triangle of A that is not stored holds NaN."""
    n, T = 16384, 1024
    configure(lib, T=T, nstreams=4, arena_gb=12.0, **AUTO)
    A, ka = pinned(n, n, 17, synth.MAT_A)
    B, kb = pinned(n, n, 17, synth.MAT_B)
    C, kc = pinned(n, n, 17, synth.MAT_C)
    for j in range(n):                                    # poison the other triangle column by column
        if uplo == blasx.Lower:
            A[:j, j] = np.nan
        else:
            A[j + 1:, j] = np.nan
    dt = timed(lambda: lib.dsymm(blasx.ColMajor, side, uplo, n, n, 1.0, A, n, B, n, 1.0, C, n))
    st = report("DSYMM %s N=16384" % ("L/L" if side == blasx.Left else "R/U"), lib, 2.0 * n ** 3, dt)
    nt = n // T
    assert st["tasks"] == nt * nt and st["tile_steps"] == nt ** 3
    assert st["evictions"] == 0 and st["bytes_d2h"] == 8 * n * n
    assert st["bytes_h2d"] == 8 * T * T * (nt * (nt + 1) // 2 + 2 * nt * nt)     # every stored tile exactly once
    rng = np.random.default_rng(17)
    before = c_before(17, synth.MAT_C, n)

    def sym_rows(idx):            # rows idx of the full symmetric matrix (which are also its columns)
        out = np.empty((len(idx), n))
        for q, i in enumerate(idx):
            if uplo == blasx.Lower:
                out[q, :i + 1] = A[i, :i + 1]
                out[q, i + 1:] = A[i + 1:, i]
            else:
                out[q, :i] = A[:i, i]
                out[q, i:] = A[i, i:]
        return out

    worst = 0.0
    for (ti, tj) in synth.sample_tiles(nt, nt, 32, 17):
        rows, cols = sampled_positions(T, T, T, rng)
        gi, gj = np.array(rows) + ti * T, np.array(cols) + tj * T
        got = np.asarray(C)[np.ix_(gi, gj)]
        c0 = before(gi, gj)
        want = np.asfortranarray(c0)
        if side == blasx.Left:
            x, y = np.asfortranarray(sym_rows(gi)), np.asfortranarray(B[:, gj])
            ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, x, y, 1.0, want)
            bound = elem_bound(norms(x, 1), norms(y, 0), 1.0, c0)
        else:
            x, y = np.asfortranarray(B[gi, :]), np.asfortranarray(sym_rows(gj))
            ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, x, y, 1.0, want)
            bound = elem_bound(norms(x, 1), norms(y, 1), 1.0, c0)
        worst = max(worst, assert_close(got, want, bound, TOL64, (ti, tj)))
    assert worst < TOL64, worst
    # every element of four whole tiles: block rows (columns) of the full symmetric matrix are put together from the
    # stored triangle here, the product is the oracle's
    for (ti, tj) in [(0, 0), (nt - 1, nt - 1), (nt - 1, 0), (3, 9)]:
        r0, c0_ = ti * T, tj * T
        before_t = synth.block(17, synth.MAT_C, n, r0, c0_, T, T)
        want = np.array(before_t, order="F")
        if side == blasx.Left:
            x, y = np.asfortranarray(sym_rows(range(r0, r0 + T))), B[:, c0_:c0_ + T]
            ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, x, y, 1.0, want)
            bound = elem_bound(norms(x, 1), norms(y, 0), 1.0, before_t)
        else:
            x, y = B[r0:r0 + T, :], np.asfortranarray(sym_rows(range(c0_, c0_ + T)))
            ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, x, y, 1.0, want)
            bound = elem_bound(norms(x, 1), norms(y, 1), 1.0, before_t)
        assert_close(np.asarray(C)[r0:r0 + T, c0_:c0_ + T], want, bound, TOL64, ("whole", ti, tj))


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS[1::3])
def test_wide_schedule_dtrsm_full_compare_and_residual(lib, side, uplo, trans, diag):
    """The triangular solve in the wide schedule (14 x 11 ragged tiles), compared element by element and by residual.
    Half of the cases with the right-hand sides in three staggered panels, two rounds apart (what large solves do)."""
    M, N = 1700, 1330
    stagger = dict(stagger_panels=3, stagger_lag=2) if (side + uplo + trans + diag) % 2 else dict(stagger_lag=-1)
    configure(lib, T=128, arena_gb=0.5, **dict(AUTO, **stagger))
    n = M if side == blasx.Left else N
    A, ka = triangular(n, 33, uplo, diag)
    B, kb = pinned(M, N, 33, 1)
    B0 = np.array(B, order="F")
    want = np.array(B, order="F")
    lib.dtrsm(blasx.ColMajor, side, uplo, trans, diag, M, N, -1.3, A, n, B, M)
    assert lib.get_option("last_wide") == 1
    ref.trsm(ref.ColMajor, side, uplo, trans, diag, -1.3, np.asarray(A), want)
    X = np.array(B, order="F")
    assert np.all(np.isfinite(X))
    assert relerr(X, want) < TOL64
    assert_trsm_residual(side, uplo, trans, diag, A, X, B0, -1.3, TOL64)


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS[2::3])
def test_wide_schedule_dtrmm_full_compare(lib, side, uplo, trans, diag):
    """The in-place triangular product in the wide schedule (14 x 13 ragged tiles): all panels pinned at once."""
    M, N = 1700, 1600
    stagger = dict(stagger_panels=3, stagger_lag=2) if (side + uplo + trans + diag) % 2 else dict(stagger_lag=-1)
    configure(lib, T=128, arena_gb=0.5, **dict(AUTO, **stagger))
    A, ka = triangular(M if side == blasx.Left else N, 34, uplo, diag)
    B, kb = pinned(M, N, 34, 1)
    want = np.array(B, order="F")
    B0 = np.array(B, order="F")
    lib.dtrmm(blasx.ColMajor, side, uplo, trans, diag, M, N, 0.9, A, A.shape[0], B, M)
    assert lib.get_option("last_wide") == 1
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 0.9, np.asarray(A), want)
    assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, 0.9), TOL64)
    assert lib.get_stats()["bytes_h2d"] >= 8 * M * N


# ------------------------------------------------------------------ integer inputs: bit for bit --
# Entries in {-2..2}: every product and every partial sum is an integer far below 2^53 (2^24 in single
# precision), so any order of summation gives the same bits and the oracle's result is THE result.  A tile,
# macro-tile, slab or chain boundary handled wrongly shows as a mismatch, however small its effect.

def int_pinned(rows, cols, seed, mat, dtype=np.float64):
    return pinned(rows, cols, seed, mat, dtype=dtype, integers=True)


@pytest.mark.parametrize("ta,tb,ktiles", [(blasx.NoTrans, blasx.NoTrans, 11), (blasx.Trans, blasx.NoTrans, 11), (blasx.NoTrans, blasx.Trans, 11),
                                          (blasx.Trans, blasx.Trans, 11), (blasx.NoTrans, blasx.NoTrans, 16), (blasx.NoTrans, blasx.NoTrans, 19)])
def test_dgemm_integer_exact_wide_schedule_tile_1024_fast_path(lib, ta, tb, ktiles):
    """The launch configuration bench.py times (T = 1024, all tasks advance together, unpredicated kernel, C tiles
    arrive late), rounds of 3+4+4, 2+6+8 and 3+8+8 k-tiles."""
    T = 1024
    M, N, K = 2 * T, 3 * T, ktiles * T
    configure(lib, T=T, arena_gb=2.0, **AUTO)
    A, ka = int_pinned(*((M, K) if ta == blasx.NoTrans else (K, M)), 50, 0)
    B, kb = int_pinned(*((K, N) if tb == blasx.NoTrans else (N, K)), 50, 1)
    C, kc = int_pinned(M, N, 50, 2)
    want = np.array(C, order="F")
    lib.dgemm(blasx.ColMajor, ta, tb, M, N, K, 2.0, A, A.shape[0], B, B.shape[0], -1.0, C, M)
    assert lib.get_option("last_wide") == 1 and lib.get_option("last_kchain") == (4 if ktiles == 11 else 8)
    ref.gemm(ref.ColMajor, ta, tb, 2.0, np.asarray(A), np.asarray(B), -1.0, want)
    assert np.array_equal(np.asarray(C), want)


@pytest.mark.parametrize("schedule", ["grouped", "wide"])
def test_symmetric_and_triangular_routines_integer_exact(lib, schedule):
    """DSYRK, DSYR2K, DSYMM and DTRMM on tile-aligned integer matrices (unpredicated and masked kernels), both schedules."""
    T = 256
    N, K = 5 * T, 12 * T
    configure(lib, T=T, arena_gb=1.0, **(AUTO if schedule == "wide" else dict(group=4, kchain=3)))
    wide = 1 if schedule == "wide" else 0
    A, ka = int_pinned(N, K, 51, 0)
    B, kb = int_pinned(N, K, 51, 1)
    for uplo, trans in ((blasx.Lower, blasx.NoTrans), (blasx.Upper, blasx.Trans)):
        C, kc = int_pinned(N, N, 51, 2)
        want = np.array(C, order="F")
        a, b = (A, B) if trans == blasx.NoTrans else (np.asfortranarray(np.asarray(A).T), np.asfortranarray(np.asarray(B).T))
        if trans == blasx.Trans:
            (a_p, k1), (b_p, k2) = blasx.pinned_matrix(K, N), blasx.pinned_matrix(K, N)
            a_p[...], b_p[...] = a, b
            a, b = a_p, b_p
        lib.dsyrk(blasx.ColMajor, uplo, trans, N, K, -1.0, a, a.shape[0], 2.0, C, N)
        assert lib.get_option("last_wide") == wide
        ref.syrk(ref.ColMajor, uplo, trans, -1.0, np.asarray(a), 2.0, want)
        assert np.array_equal(np.asarray(C), want), ("syrk", uplo, trans)
        lib.dsyr2k(blasx.ColMajor, uplo, trans, N, K, 1.0, a, a.shape[0], b, b.shape[0], -1.0, C, N)
        assert lib.get_option("last_wide") == wide
        ref.syr2k(ref.ColMajor, uplo, trans, 1.0, np.asarray(a), np.asarray(b), -1.0, want)
        assert np.array_equal(np.asarray(C), want), ("syr2k", uplo, trans)
    n = 12 * T
    S, ks = int_pinned(n, n, 52, 0)
    X, kx = int_pinned(n, 3 * T, 52, 1)
    for side, uplo in ((blasx.Left, blasx.Lower), (blasx.Right, blasx.Upper)):
        Sp, kp = blasx.pinned_matrix(n, n)
        Sp[...] = np.asarray(S)
        Sp[np.triu_indices(n, 1) if uplo == blasx.Lower else np.tril_indices(n, -1)] = np.nan      # never read
        Xs, kxs = (X, kx) if side == blasx.Left else blasx.pinned_matrix(3 * T, n)
        if side == blasx.Right:
            Xs[...] = np.asarray(X).T
        Y, ky = int_pinned(Xs.shape[0], Xs.shape[1], 52, 2)
        want = np.array(Y, order="F")
        lib.dsymm(blasx.ColMajor, side, uplo, Xs.shape[0], Xs.shape[1], 1.0, Sp, n, Xs, Xs.shape[0], 1.0, Y, Xs.shape[0])
        assert lib.get_option("last_wide") == wide
        ref.symm(ref.ColMajor, side, uplo, 1.0, np.asarray(Sp), np.asarray(Xs), 1.0, want)
        assert np.array_equal(np.asarray(Y), want), ("symm", side, uplo)
    for side, uplo, trans, diag in ((blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit), (blasx.Right, blasx.Upper, blasx.Trans, blasx.Unit),
                                    (blasx.Left, blasx.Upper, blasx.NoTrans, blasx.Unit), (blasx.Right, blasx.Lower, blasx.NoTrans, blasx.NonUnit)):
        Tp, kt = blasx.pinned_matrix(n, n)
        Tp[...] = np.asarray(S)
        Tp[np.triu_indices(n, 1) if uplo == blasx.Lower else np.tril_indices(n, -1)] = np.nan
        if diag == blasx.Unit:
            Tp[np.diag_indices(n)] = np.nan
        Bs, kbs = blasx.pinned_matrix(n, 3 * T) if side == blasx.Left else blasx.pinned_matrix(3 * T, n)
        Bs[...] = np.asarray(X) if side == blasx.Left else np.asarray(X).T
        want = np.array(Bs, order="F")
        lib.dtrmm(blasx.ColMajor, side, uplo, trans, diag, Bs.shape[0], Bs.shape[1], -2.0, Tp, n, Bs, Bs.shape[0])
        assert lib.get_option("last_wide") == wide
        ref.trmm(ref.ColMajor, side, uplo, trans, diag, -2.0, np.asarray(Tp), want)
        assert np.array_equal(np.asarray(Bs), want), ("trmm", side, uplo, trans, diag)


@pytest.mark.parametrize("schedule", ["grouped", "wide"])
@pytest.mark.parametrize("ta,tb", [(blasx.NoTrans, blasx.NoTrans), (blasx.Trans, blasx.NoTrans), (blasx.NoTrans, blasx.Trans)])
def test_neighbouring_tiles_share_an_inbound_copy_integer_exact(lib, schedule, ta, tb):
    """Whole tiles that lie side by side in a block row of a host matrix travel in one strided copy ("merge" tiles at
    most) when they go to neighbouring slots.  The copy engine then sees fewer copies than tiles; bytes, tile counts
    and results (integer inputs: bit for bit) are those of one copy per tile.  Both schedules; in the grouped one
    also with C fetched for the first launch and in queue order."""
    T = 256
    M, N, K = 8 * T, 8 * T, 12 * T
    A, ka = int_pinned(M if ta == blasx.NoTrans else K, K if ta == blasx.NoTrans else M, 61, 0)
    B, kb = int_pinned(K if tb == blasx.NoTrans else N, N if tb == blasx.NoTrans else K, 61, 1)
    C0, kc = int_pinned(M, N, 61, 2)
    want = np.array(C0, order="F")
    ref.gemm(ref.ColMajor, ta, tb, 2.0, np.asarray(A), np.asarray(B), -1.0, want)
    variants = [dict(merge=1), dict(merge=4), dict(merge=8), dict(merge=0)]
    if schedule == "grouped":
        variants += [dict(merge=4, late_c=0), dict(merge=4, row_order=0), dict(merge=8, late_c=0, row_order=0, kchain=3)]
    transfers = []
    for v in variants:
        configure(lib, T=T, arena_gb=1.0, **dict(AUTO if schedule == "wide" else dict(group=4, kchain=0), **v))
        C, kcc = blasx.pinned_matrix(M, N)
        C[...] = np.asarray(C0)
        lib.dgemm(blasx.ColMajor, ta, tb, M, N, K, 2.0, A, A.shape[0], B, B.shape[0], -1.0, C, M)
        assert lib.get_option("last_wide") == (1 if schedule == "wide" else 0)
        assert np.array_equal(np.asarray(C), want), (schedule, v)
        st = lib.get_stats()
        assert st["copies_h2d"] == 64 + 2 * 96 and st["bytes_h2d"] == 8 * (M * K + K * N + M * N), (v, st)
        assert st["steps_general"] == 0
        transfers.append(st["transfers_h2d"])
    print("inbound copies for 256 tiles:", list(zip([str(v) for v in variants], transfers)), flush=True)
    assert transfers[0] == 256
    assert all(t <= 0.7 * 256 for t in transfers[1:]), transfers


@pytest.mark.parametrize("ta,tb,T", [(blasx.NoTrans, blasx.Trans, 1024), (blasx.Trans, blasx.NoTrans, 512), (blasx.NoTrans, blasx.NoTrans, 2048)])
def test_sgemm_integer_exact(lib, ta, tb, T):
    """Single precision: entries in {-2..2} and K <= 22528 keep every partial sum below 2^24, so float32 is exact too."""
    M, N, K = 2 * T, 2 * T, 11 * T
    configure(lib, T=T, arena_gb=2.0, **AUTO)
    f32 = np.float32
    A, ka = int_pinned(*((M, K) if ta == blasx.NoTrans else (K, M)), 53, 0, dtype=f32)
    B, kb = int_pinned(*((K, N) if tb == blasx.NoTrans else (N, K)), 53, 1, dtype=f32)
    C, kc = int_pinned(M, N, 53, 2, dtype=f32)
    want = np.array(C, order="F")
    lib.sgemm(blasx.ColMajor, ta, tb, M, N, K, 2.0, A, A.shape[0], B, B.shape[0], -1.0, C, M)
    assert lib.get_option("last_wide") == 1
    ref.gemm(ref.ColMajor, ta, tb, 2.0, np.asarray(A), np.asarray(B), -1.0, want)
    assert np.array_equal(np.asarray(C), want)


# ------------------------------------------------------------------ boundary: streams, time profile --

def test_set_streams_between_calls(lib):
    """blasx_set_streams re-roles the streams of the current initialisation: 2, 3 and 4 streams give the same bits."""
    n = 1536
    configure(lib, T=256, nstreams=4, arena_gb=0.5)
    A, ka = int_pinned(n, n, 54, 0)
    B, kb = int_pinned(n, n, 54, 1)
    want = np.zeros((n, n), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, np.asarray(A), np.asarray(B), 0.0, want)
    for ns in (2, 3, 4, 2, 0):
        lib.set_streams(ns)
        assert lib.get_option("streams") == (ns or 4)
        C, kc = blasx.pinned_matrix(n, n)
        C[...] = np.nan
        lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
        assert np.array_equal(np.asarray(C), want), ns
    assert lib._lib.blasx_set_streams(5) == 4 and lib._lib.blasx_set_streams(1) == 4


def test_time_profile_of_a_call(lib):
    """Option profile = 2: the call's time on the device dissected into kernels, copies that no kernel hides, and the
    rest (Section V.A); and the host's time into issuing and waiting."""
    n, T = 8192, 1024
    configure(lib, T=T, nstreams=4, arena_gb=4.0, profile=2, **AUTO)
    A, ka = pinned(n, n, 55, 0)
    B, kb = pinned(n, n, 55, 1)
    C, kc = pinned(n, n, 55, 2)
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)      # warm-up
    lib.reset_stats()
    dt = timed(lambda: lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n))
    st = lib.get_stats()
    lib.set_option("profile", 0)
    busy, comm, span = st["t_kernel_busy_s"], st["t_copy_unoverlapped_s"], st["t_device_span_s"]
    print("\n[result] time profile DGEMM N=8192: wall %.2f ms, device span %.2f ms = kernels %.2f + unhidden copies %.2f + other %.2f; "
          "host issuing %.2f ms, waiting %.2f ms" % (dt * 1e3, span * 1e3, busy * 1e3, comm * 1e3, (span - busy - comm) * 1e3,
                                                     st["t_issue_s"] * 1e3, st["t_wait_s"] * 1e3), flush=True)
    assert 0 < busy <= span and 0 <= comm <= span and busy + comm <= span * (1 + 1e-6)
    assert span <= dt and span > 0.5 * dt
    assert abs(st["t_total_s"] - st["t_issue_s"] - st["t_wait_s"]) < 1e-6
    # the kernels of this call need 1.1 TFLOP / 78.6 TFLOP/s = 14 ms at the very least, its copies 1.6 GB / 57 GB/s = 28 ms:
    # so at least half of the copy time cannot be under a kernel, and the device span is mostly copies
    assert busy >= 2.0 * n ** 3 / 78.6e12 and busy + comm >= 3 * 8 * n * n / 64e9
    assert st["t_kernel_s"] >= busy * (1 - 1e-6)          # launches never overlap each other: one compute stream


def test_priorities_save_tile_fetches_under_a_small_cache(lib):
    """Alg. 1 lines 10-15, Eq. 2 on the device: a cache of 12 tiles, one task running, a station of 4 tasks whose
    priorities (cached operand tiles) are refreshed whenever a task comes in.  An 8 x 8-tile product with 4 k-tiles
    then fetches fewer tiles than with the priorities switched off (queue order); both results are exact."""
    T, nt, nk = 256, 8, 4
    n = nt * T
    A, ka = int_pinned(n, nk * T, 56, 0)
    B, kb = int_pinned(nk * T, n, 56, 1)
    want = np.zeros((n, n), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.asarray(A), np.asarray(B), 0.0, want)
    misses = {}
    for prio in (0, 1):
        configure(lib, T=T, arena_gb=0.25, cap_bytes=12 * T * T * 8, group=1, rs=4, kchain=1, priority=prio, sb_rows=2, sb_cols=2, shells=0)
        C, kc = blasx.pinned_matrix(n, n)
        C[...] = np.nan
        lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, nk * T, 1.0, A, n, B, nk * T, 0.0, C, n)
        assert np.array_equal(np.asarray(C), want)
        st = lib.get_stats()
        assert st["peak_slots"] <= 12 and st["misses"] == 2 * nt * nk + st["refetches"]
        misses[prio] = st["misses"]
    lib.set_option("priority", 1)
    lib.set_option("shells", 1)
    print("\n[result] tile fetches of an 8 x 8 x 4-tile DGEMM under a 12-tile cache: %d in queue order, %d with Eq. 2 priorities"
          % (misses[0], misses[1]), flush=True)
    assert misses[1] < misses[0], misses


# ------------------------------------------------------------------ automatic tile size --

@pytest.mark.parametrize("n,expect,group", [(1000, 1008, 2), (4096, 1024, 2), (8192, 1024, 4)])  # all below the wide threshold
def test_auto_tile_dgemm_sampled(lib, n, expect, group):
    """blasx_set_tile(0) and group 0: tile and running set are chosen per call; same parity bar as fixed ones."""
    configure(lib, T=0, nstreams=4, arena_gb=4.0, group=0)
    A, ka = pinned(n, n, 19, synth.MAT_A)
    B, kb = pinned(n, n, 19, synth.MAT_B)
    C, kc = pinned(n, n, 19, synth.MAT_C)
    dt = timed(lambda: lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, n, B, n, 1.0, C, n))
    T = lib.get_option("last_tile")
    report("auto tile DGEMM NT N=%d -> T=%d" % (n, T), lib, 2.0 * n ** 3, dt)
    assert T == expect and lib.get_option("last_group") == group
    check_gemm_sampled(blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, B, 1.0, c_before(19, synth.MAT_C, n), C, T, 19, TOL64)
    check_gemm_whole_tiles(blasx.NoTrans, blasx.Trans, n, n, n, 1.0, A, B, 1.0, (19, synth.MAT_C), C, T, 16, 19, TOL64)


# ------------------------------------------------------------------ persistent tile cache --

def test_persistent_cache_repeated_products_with_resident_weights(lib):
    """The application pattern of Section V.C: one weight matrix W (16384^2), a stream of activation batches X_b
    (16384 x 4096).  With the persistent cache W crosses the link once; every later call copies its batch only."""
    n, nb, T = 16384, 4096, 1024
    configure(lib, T=T, nstreams=4, arena_gb=8.0, persist=1)
    W, kw = pinned(n, n, 18, synth.MAT_A)
    X = [pinned(n, nb, 18 + b, synth.MAT_B) for b in range(3)]
    Y, ky = blasx.pinned_matrix(n, nb)
    times, stats = [], []
    for b in range(3):
        lib.reset_stats()
        times.append(timed(lambda: lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, nb, n, 1.0, W, n, X[b][0], n, 0.0, Y, n)))
        stats.append(report("persistent W: batch %d, DGEMM 16384x4096x16384" % b, lib, 2.0 * n * nb * n, times[-1]))
        check_gemm_sampled(blasx.NoTrans, blasx.NoTrans, n, nb, n, 1.0, W, X[b][0], 0.0, lambda gi, gj: np.zeros((len(gi), len(gj))),
                           Y, T, 18 + b, TOL64)
    assert stats[0]["bytes_h2d"] == 8 * (n * n + n * nb)
    assert stats[1]["bytes_h2d"] == 8 * n * nb and stats[2]["bytes_h2d"] == 8 * n * nb
    assert stats[1]["misses"] == (n // T) * (nb // T)
    # the host changes W: after the invalidation the new values are used
    W[:, :1] = 0.0
    lib.reset_stats()
    lib.invalidate_matrix(W, n, n, 1, 8)            # first column only: one block column of tiles is dropped
    lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, nb, n, 1.0, W, n, X[0][0], n, 0.0, Y, n)
    st = lib.get_stats()
    assert st["invalidations"] == n // T and st["bytes_h2d"] == 8 * n * T      # batch 0 is still cached as well
    check_gemm_sampled(blasx.NoTrans, blasx.NoTrans, n, nb, n, 1.0, W, X[0][0], 0.0, lambda gi, gj: np.zeros((len(gi), len(gj))),
                       Y, T, 21, TOL64)
    check_gemm_whole_tiles(blasx.NoTrans, blasx.NoTrans, n, nb, n, 1.0, W, X[0][0], 0.0, None, Y, T, 4, 21, TOL64)
    lib.set_option("persist", 0)


# ------------------------------------------------------------------ single-precision variants --

def test_single_precision_syrk_trmm_trsm(lib):
    """The fp32 entry points share the task builders and kernels of the fp64 ones."""
    N, K = 900, 640
    configure(lib, T=256, arena_gb=0.25, group=6)
    A, ka = pinned(N, K, 12, 0, dtype=np.float32)
    C, kc = pinned(N, N, 12, 2, dtype=np.float32)
    want = np.array(C, order="F")
    C0 = np.array(C, order="F")
    lib.ssyrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, N, K, 1.0, A, N, 1.0, C, N)
    ref.syrk(ref.ColMajor, ref.Lower, ref.NoTrans, 1.0, np.asarray(A), 1.0, want)
    assert_close(C, want, elem_bound(norms(A, 1), norms(A, 1), 1.0, C0, single=True, want=want) + square_sums(norms(A, 1), K, single=True), TOL32)
    M, Nb = 768, 520
    T64, kt = triangular(M, 13, blasx.Upper, blasx.NonUnit)
    T32, k32 = blasx.pinned_matrix(M, M, dtype=np.float32)
    T32[...] = np.asarray(T64).astype(np.float32)
    B, kb = pinned(M, Nb, 13, 1, dtype=np.float32)
    want = np.array(B, order="F")
    B0 = np.array(B, order="F")
    lib.strmm(blasx.ColMajor, blasx.Left, blasx.Upper, blasx.Trans, blasx.NonUnit, M, Nb, 1.0, T32, M, B, M)
    ref.trmm(ref.ColMajor, ref.Left, ref.Upper, ref.Trans, ref.NonUnit, 1.0, np.asarray(T32), want)
    assert_close(B, want, trmm_bound(blasx.Left, blasx.Upper, blasx.Trans, blasx.NonUnit, T32, B0, 1.0, single=True, want=want), TOL32)
    synth.fill(B, 13, 1)
    want = np.array(B, order="F")
    B0 = np.array(B, order="F")
    lib.strsm(blasx.ColMajor, blasx.Left, blasx.Upper, blasx.NoTrans, blasx.NonUnit, M, Nb, 1.0, T32, M, B, M)
    ref.trsm(ref.ColMajor, ref.Left, ref.Upper, ref.NoTrans, ref.NonUnit, 1.0, np.asarray(T32), want)
    assert relerr(B, want) < TOL32
    assert_trsm_residual(blasx.Left, blasx.Upper, blasx.NoTrans, blasx.NonUnit, T32, B, B0, 1.0, TOL32, single=True)


# ------------------------------------------------------------------ seeded random problems --

@pytest.mark.parametrize("seed", range(36))
def test_seeded_random_problems_every_routine_and_schedule(lib, seed):
    """Routine, flags, ragged extents, tile size, schedule options and scalars drawn from a seeded generator; every
    element compared with the oracle.  The k extents reach 30 tiles, so the wide schedule's rounds come out in every
    shape (left-over steps first, a split first round, two rounds only)."""
    rng = np.random.default_rng(1000 + seed)
    routine = ("gemm", "syrk", "syr2k", "symm", "trmm", "trsm")[seed % 6]
    T = int(rng.choice([128, 256, 208]))      # 208: no multiple of the macro-tile edge, the bounds-checked kernel
    opts = dict(group=int(rng.choice([0, 4, 16])), kchain=int(rng.choice([0, 0, 3, 8])), wide=int(rng.choice([0, 2, 12])),
                ramp=int(rng.choice([0, 0, 1, 8])))
    # how tiles travel and when C is fetched (a generator of their own: the problems above stay what they were)
    rng2 = np.random.default_rng(5000 + seed)
    opts.update(merge=int(rng2.choice([1, 0, 4, 8])), late_c=int(rng2.choice([0, 1, 1])), row_order=int(rng2.choice([0, 1, 1])),
                stagger_panels=int(rng2.choice([1, 2, 3])), stagger_lag=int(rng2.choice([0, 1, 2, 4])), tail_cut=int(rng2.choice([0, 4, 4, 2])))
    configure(lib, T=T, arena_gb=1.5, **opts)
    uplo = int(rng.choice([blasx.Lower, blasx.Upper]))
    trans = int(rng.choice(TRANS))
    side = int(rng.choice([blasx.Left, blasx.Right]))
    diag = int(rng.choice([blasx.NonUnit, blasx.Unit]))
    alpha = float(rng.choice([1.0, -0.6, 0.0, 1.7]))
    beta = float(rng.choice([0.0, 1.0, -1.3]))
    M, N = int(rng.integers(200, 1500)), int(rng.integers(200, 1500))
    K = int(rng.integers(100, 30 * T))
    tag = "%s T=%d %s M=%d N=%d K=%d uplo=%d trans=%d side=%d diag=%d alpha=%g beta=%g" % (routine, T, opts, M, N, K, uplo, trans, side, diag, alpha, beta)
    print(tag, flush=True)
    if routine == "gemm":
        ta, tb = trans, int(rng.choice(TRANS))
        A, ka = pinned(M if ta == blasx.NoTrans else K, K if ta == blasx.NoTrans else M, seed, 0)
        B, kb = pinned(K if tb == blasx.NoTrans else N, N if tb == blasx.NoTrans else K, seed, 1)
        C, kc = pinned(M, N, seed, 2)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        lib.dgemm(blasx.ColMajor, ta, tb, M, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C, M)
        ref.gemm(ref.ColMajor, ta, tb, alpha, np.asarray(A), np.asarray(B), beta, want)
        assert_close(C, want, elem_bound(norms(op(A, ta), 1), norms(op(B, tb), 0), alpha, beta * C0), TOL64, tag)
    elif routine in ("syrk", "syr2k"):
        K = min(K, 12 * T)
        A, ka = pinned(N if trans == blasx.NoTrans else K, K if trans == blasx.NoTrans else N, seed, 0)
        B, kb = pinned(A.shape[0], A.shape[1], seed, 1)
        C, kc = pinned(N, N, seed, 2)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        ra, rb = norms(op(A, trans), 1), norms(op(B, trans), 1)
        if routine == "syrk":
            lib.dsyrk(blasx.ColMajor, uplo, trans, N, K, alpha, A, A.shape[0], beta, C, N)
            ref.syrk(ref.ColMajor, uplo, trans, alpha, np.asarray(A), beta, want)
            bound = elem_bound(ra, ra, alpha, beta * C0) + square_sums(ra, K, alpha)
        else:
            lib.dsyr2k(blasx.ColMajor, uplo, trans, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C, N)
            ref.syr2k(ref.ColMajor, uplo, trans, alpha, np.asarray(A), np.asarray(B), beta, want)
            bound = elem_bound(ra, rb, alpha, beta * C0) + elem_bound(rb, ra, alpha)
        assert_close(C, want, bound, TOL64, tag)
    elif routine == "symm":
        n = M if side == blasx.Left else N
        A, ka = pinned(n, n, seed, 0)
        B, kb = pinned(M, N, seed, 1)
        C, kc = pinned(M, N, seed, 2)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        lib.dsymm(blasx.ColMajor, side, uplo, M, N, alpha, A, n, B, M, beta, C, M)
        ref.symm(ref.ColMajor, side, uplo, alpha, np.asarray(A), np.asarray(B), beta, want)
        S = sym_matrix(A, uplo)
        if side == blasx.Left:
            bound = elem_bound(norms(S, 1), norms(B, 0), alpha, beta * C0)
        else:
            bound = elem_bound(norms(B, 1), norms(S, 0), alpha, beta * C0)
        assert_close(C, want, bound, TOL64, tag)
    else:
        n = M if side == blasx.Left else N
        A, ka = triangular(n, seed, uplo, diag)
        B, kb = pinned(M, N, seed, 1)
        B0 = np.array(B, order="F")
        want = np.array(B, order="F")
        alpha = alpha if alpha != 0.0 else 0.9
        if routine == "trmm":
            lib.dtrmm(blasx.ColMajor, side, uplo, trans, diag, M, N, alpha, A, n, B, M)
            ref.trmm(ref.ColMajor, side, uplo, trans, diag, alpha, np.asarray(A), want)
            assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, alpha), TOL64, tag)
        else:
            lib.dtrsm(blasx.ColMajor, side, uplo, trans, diag, M, N, alpha, A, n, B, M)
            assert_trsm_residual(side, uplo, trans, diag, A, B, B0, alpha, TOL64, tag)


@pytest.mark.parametrize("seed", range(18))
def test_seeded_random_problems_single_precision(lib, seed):
    """The same in single precision (tile-aligned and ragged extents, so both the fast and the general kernel run)."""
    rng = np.random.default_rng(2000 + seed)
    routine = ("gemm", "syrk", "syr2k", "symm", "trmm", "trsm")[seed % 6]
    T = int(rng.choice([256, 512, 336]))      # 336: the bounds-checked kernel
    opts = dict(group=int(rng.choice([0, 4, 16])), kchain=int(rng.choice([0, 0, 3])), wide=int(rng.choice([0, 2, 12])))
    configure(lib, T=T, arena_gb=1.5, **opts)
    uplo = int(rng.choice([blasx.Lower, blasx.Upper]))
    trans = int(rng.choice(TRANS))
    side = int(rng.choice([blasx.Left, blasx.Right]))
    diag = int(rng.choice([blasx.NonUnit, blasx.Unit]))
    alpha = float(rng.choice([1.0, -0.6, 1.7]))
    beta = float(rng.choice([0.0, 1.0, -1.3]))
    aligned = bool(rng.integers(0, 2))
    M = int(rng.integers(1, 5)) * T if aligned else int(rng.integers(200, 1500))
    N = int(rng.integers(1, 5)) * T if aligned else int(rng.integers(200, 1500))
    K = int(rng.integers(1, 20)) * T if aligned else int(rng.integers(100, 20 * T))
    tag = "%s T=%d %s M=%d N=%d K=%d uplo=%d trans=%d side=%d diag=%d alpha=%g beta=%g" % (routine, T, opts, M, N, K, uplo, trans, side, diag, alpha, beta)
    print(tag, flush=True)
    f32 = np.float32

    def single(a64):
        a, owner = blasx.pinned_matrix(a64.shape[0], a64.shape[1], dtype=f32)
        a[...] = np.asarray(a64).astype(f32)
        return a, owner

    if routine == "gemm":
        ta, tb = trans, int(rng.choice(TRANS))
        A, ka = pinned(M if ta == blasx.NoTrans else K, K if ta == blasx.NoTrans else M, seed, 0, dtype=f32)
        B, kb = pinned(K if tb == blasx.NoTrans else N, N if tb == blasx.NoTrans else K, seed, 1, dtype=f32)
        C, kc = pinned(M, N, seed, 2, dtype=f32)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        lib.sgemm(blasx.ColMajor, ta, tb, M, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C, M)
        ref.gemm(ref.ColMajor, ta, tb, alpha, np.asarray(A), np.asarray(B), beta, want)
        assert_close(C, want, elem_bound(norms(op(A, ta), 1), norms(op(B, tb), 0), alpha, beta * C0, single=True, want=want), TOL32, tag)
    elif routine in ("syrk", "syr2k"):
        K = min(K, 12 * T)
        A, ka = pinned(N if trans == blasx.NoTrans else K, K if trans == blasx.NoTrans else N, seed, 0, dtype=f32)
        B, kb = pinned(A.shape[0], A.shape[1], seed, 1, dtype=f32)
        C, kc = pinned(N, N, seed, 2, dtype=f32)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        ra, rb = norms(op(A, trans), 1), norms(op(B, trans), 1)
        if routine == "syrk":
            lib.ssyrk(blasx.ColMajor, uplo, trans, N, K, alpha, A, A.shape[0], beta, C, N)
            ref.syrk(ref.ColMajor, uplo, trans, alpha, np.asarray(A), beta, want)
            bound = elem_bound(ra, ra, alpha, beta * C0, single=True, want=want) + square_sums(ra, K, alpha, single=True)
        else:
            lib.ssyr2k(blasx.ColMajor, uplo, trans, N, K, alpha, A, A.shape[0], B, B.shape[0], beta, C, N)
            ref.syr2k(ref.ColMajor, uplo, trans, alpha, np.asarray(A), np.asarray(B), beta, want)
            bound = elem_bound(ra, rb, alpha, beta * C0, single=True, want=want) + elem_bound(rb, ra, alpha)
        assert_close(C, want, bound, TOL32, tag)
    elif routine == "symm":
        n = M if side == blasx.Left else N
        A, ka = pinned(n, n, seed, 0, dtype=f32)
        B, kb = pinned(M, N, seed, 1, dtype=f32)
        C, kc = pinned(M, N, seed, 2, dtype=f32)
        want = np.array(C, order="F")
        C0 = np.array(C, order="F")
        lib.ssymm(blasx.ColMajor, side, uplo, M, N, alpha, A, n, B, M, beta, C, M)
        ref.symm(ref.ColMajor, side, uplo, alpha, np.asarray(A), np.asarray(B), beta, want)
        S = sym_matrix(A, uplo)
        if side == blasx.Left:
            bound = elem_bound(norms(S, 1), norms(B, 0), alpha, beta * C0, single=True, want=want)
        else:
            bound = elem_bound(norms(B, 1), norms(S, 0), alpha, beta * C0, single=True, want=want)
        assert_close(C, want, bound, TOL32, tag)
    else:
        n = M if side == blasx.Left else N
        A64, k64 = triangular(n, seed, uplo, diag)
        A, ka = single(A64)
        B, kb = pinned(M, N, seed, 1, dtype=f32)
        want = np.array(B, order="F")
        B0 = np.array(B, order="F")
        if routine == "trmm":
            lib.strmm(blasx.ColMajor, side, uplo, trans, diag, M, N, alpha, A, n, B, M)
            ref.trmm(ref.ColMajor, side, uplo, trans, diag, alpha, np.asarray(A), want)
            assert_close(B, want, trmm_bound(side, uplo, trans, diag, A, B0, alpha, single=True, want=want), TOL32, tag)
        else:
            lib.strsm(blasx.ColMajor, side, uplo, trans, diag, M, N, alpha, A, n, B, M)
            ref.trsm(ref.ColMajor, side, uplo, trans, diag, alpha, np.asarray(A), want)
            assert np.all(np.isfinite(np.asarray(B))) and relerr(B, want) < TOL32, tag
            assert_trsm_residual(side, uplo, trans, diag, A, B, B0, alpha, TOL32, tag, single=True)
