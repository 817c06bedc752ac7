"""Pins for the CPU oracle (no GPU).

The paper prints no worked numeric example, so the oracle is pinned to what
the mathematics fixes: exact rational brute force on tiny inputs, closed forms
(identity, diagonal, rank-1), integer-exact inputs, known-solution recovery for
TRSM, untouched-triangle and not-read (NaN poison) rules, and a compensated
dot product at the benchmark's inner dimension.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle as ref
import synth
from tests import exact

U = 2.0 ** -53
ORDERS = [ref.ColMajor, ref.RowMajor]
TRANS = [ref.NoTrans, ref.Trans]


def store(logical, order, pad=0, dtype=np.float64, fill=np.nan):
    """Copy a logical matrix into storage of the given order with `pad` extra ld; padding is NaN."""
    r, c = logical.shape
    if order == ref.ColMajor:
        buf = np.full((r + pad, c), fill, dtype=dtype, order="F")
    else:
        buf = np.full((r, c + pad), fill, dtype=dtype, order="C")
    view = buf[:r, :c]
    view[...] = logical
    return view


def rnd(rng, r, c):
    return rng.uniform(-1, 1, size=(r, c))


# ---------------------------------------------------------------- GEMM ----

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (5, 2, 3), (3, 7, 1), (7, 5, 7)])
def test_gemm_exact_rational_bruteforce(order, ta, tb, M, N, K):
    rng = np.random.default_rng(1000 * M + 100 * N + K + ta + 2 * tb + order)
    alpha, beta = 1.25 * rng.uniform(-1, 1), rng.uniform(-1, 1)
    A = rnd(rng, *((M, K) if ta == ref.NoTrans else (K, M)))
    B = rnd(rng, *((K, N) if tb == ref.NoTrans else (N, K)))
    C = rnd(rng, M, N)
    As, Bs, Cs = store(A, order, 2), store(B, order, 1), store(C, order, 3)
    ref.gemm(order, ta, tb, alpha, As, Bs, beta, Cs)
    Ae = exact.frac(A) if ta == ref.NoTrans else exact.transpose(exact.frac(A))
    Be = exact.frac(B) if tb == ref.NoTrans else exact.transpose(exact.frac(B))
    P, Pabs, Ce = exact.matmul(Ae, Be), exact.abs_matmul(Ae, Be), exact.frac(C)
    fa, fb = Fraction(alpha), Fraction(beta)
    for i in range(M):
        for j in range(N):
            want = fa * P[i][j] + fb * Ce[i][j]
            bound = (K + 4) * U * float(abs(fa) * Pabs[i][j] + abs(fb * Ce[i][j])) + 1e-300
            assert abs(Fraction(float(Cs[i, j])) - want) <= bound, (i, j)


@pytest.mark.parametrize("order", ORDERS)
def test_gemm_identity_is_exact(order):
    rng = np.random.default_rng(3)
    n, m = 9, 6
    B, C = rnd(rng, n, m), rnd(rng, n, m)
    alpha, beta = 0.5, -2.0          # powers of two: alpha*B + beta*C has one rounding
    Cs = store(C, order, 1)
    ref.gemm(order, ref.NoTrans, ref.NoTrans, alpha, store(np.eye(n), order), store(B, order, 2), beta, Cs)
    assert np.array_equal(np.asarray(Cs), alpha * B + beta * C)
    # identity on the right, transposed operand
    Cs = store(C.T.copy(), order)
    ref.gemm(order, ref.Trans, ref.NoTrans, 1.0, store(B, order), store(np.eye(n), order), 0.0, Cs)
    assert np.array_equal(np.asarray(Cs), B.T)


def test_gemm_diagonal_closed_form():
    rng = np.random.default_rng(4)
    n, m = 8, 5
    d = rng.uniform(-1, 1, n)
    B, C = rnd(rng, n, m), rnd(rng, n, m)
    alpha, beta = 0.75, 0.3
    Cs = store(C, ref.ColMajor)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, alpha, store(np.diag(d), ref.ColMajor), store(B, ref.ColMajor), beta, Cs)
    want = alpha * (d[:, None] * B) + beta * C
    assert np.max(np.abs(np.asarray(Cs) - want)) <= 4 * U * np.max(np.abs(want))


def test_gemm_rank_one_closed_form():
    x = np.array([[1.0], [-2.0], [3.0], [0.5]])
    y = np.array([[2.0, -1.0, 4.0]])
    C = np.arange(12, dtype=np.float64).reshape(4, 3)
    Cs = store(C, ref.ColMajor, 2)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 2.0, store(x, ref.ColMajor), store(y, ref.ColMajor), -1.0, Cs)
    assert np.array_equal(np.asarray(Cs), 2.0 * x @ y - C)
    # K copies of the same outer product: alpha*K*x_i*y_j exactly (small integers)
    K = 37
    A = np.repeat(x, K, axis=1)
    B = np.repeat(y, K, axis=0)
    Cs = store(np.zeros((4, 3)), ref.ColMajor)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, store(A, ref.ColMajor), store(B, ref.ColMajor), 0.0, Cs)
    assert np.array_equal(np.asarray(Cs), K * (x @ y))


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_gemm_integer_inputs_bit_exact(order, ta, tb):
    M, N, K = 13, 11, 29
    A = synth.matrix(*((M, K) if ta == ref.NoTrans else (K, M)), seed=5, mat=0, integers=True)
    B = synth.matrix(*((K, N) if tb == ref.NoTrans else (N, K)), seed=5, mat=1, integers=True)
    C = synth.matrix(M, N, seed=5, mat=2, integers=True)
    Cs = store(C, order, 1)
    ref.gemm(order, ta, tb, 2.0, store(A, order, 3), store(B, order), -3.0, Cs)
    Ai = np.asarray(A, dtype=np.int64) if ta == ref.NoTrans else np.asarray(A, dtype=np.int64).T
    Bi = np.asarray(B, dtype=np.int64) if tb == ref.NoTrans else np.asarray(B, dtype=np.int64).T
    want = 2 * (Ai @ Bi) - 3 * np.asarray(C, dtype=np.int64)
    assert np.array_equal(np.asarray(Cs), want.astype(np.float64))


def test_gemm_beta_zero_does_not_read_c_and_alpha_zero_does_not_read_ab():
    rng = np.random.default_rng(6)
    A, B = rnd(rng, 4, 3), rnd(rng, 3, 5)
    Cs = np.full((4, 5), np.nan, order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, store(A, ref.ColMajor), store(B, ref.ColMajor), 0.0, Cs)
    assert np.all(np.isfinite(Cs)) and np.allclose(Cs, A @ B, rtol=1e-14)
    C = rnd(rng, 4, 5)
    Cs = store(C, ref.ColMajor)
    nanA, nanB = np.full((4, 3), np.nan, order="F"), np.full((3, 5), np.nan, order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 0.0, nanA, nanB, 0.5, Cs)
    assert np.array_equal(np.asarray(Cs), 0.5 * C)
    # K = 0 scales C only
    Cs = store(C, ref.ColMajor)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, np.zeros((4, 0), order="F"), np.zeros((0, 5), order="F"), 2.0, Cs)
    assert np.array_equal(np.asarray(Cs), 2.0 * C)


def _two_sum(a, b):
    s = a + b
    bb = s - a
    return s, (a - (s - bb)) + (b - bb)


def _two_prod(a, b):
    # Dekker / Veltkamp splitting: exact product as hi + lo
    p = a * b
    c = 134217729.0
    ah = c * a - (c * a - a); al = a - ah
    bh = c * b - (c * b - b); bl = b - bh
    return p, ((ah * bh - p) + ah * bl + al * bh) + al * bl


def test_gemm_long_inner_dimension_against_compensated_dot():
    """At K = 32768 (the benchmark's inner dimension) the oracle's own error stays far below the 1e-13 gate."""
    K = 32768
    A = synth.matrix(3, K, seed=7, mat=0)
    B = synth.matrix(K, 2, seed=7, mat=1)
    Cs = np.zeros((3, 2), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, A, B, 0.0, Cs)
    num = den = 0.0
    for i in range(3):
        for j in range(2):
            hi = lo = 0.0
            for l in range(K):
                p, e = _two_prod(float(A[i, l]), float(B[l, j]))
                hi, e2 = _two_sum(hi, p)
                lo += e + e2
            want = hi + lo
            num += (Cs[i, j] - want) ** 2
            den += want ** 2
    assert (num / den) ** 0.5 < 2e-14


def test_sgemm_accumulates_in_double_and_rounds_once():
    rng = np.random.default_rng(8)
    M, N, K = 4, 3, 50
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    Cs = store(C, ref.ColMajor, 1, dtype=np.float32)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, store(A, ref.ColMajor, dtype=np.float32), store(B, ref.ColMajor, dtype=np.float32), 1.0, Cs)
    P = exact.matmul(exact.frac(A), exact.frac(B))
    Ce = exact.frac(C)
    for i in range(M):
        for j in range(N):
            want = float(P[i][j] + Ce[i][j])
            # one float32 rounding of an (almost) exact double: within 0.5000001 ulp_32
            assert abs(float(Cs[i, j]) - want) <= (2.0 ** -24) * 1.0001 * abs(want) + 1e-30


@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_gemm_transposed_equals_materialised_transpose(ta, tb):
    rng = np.random.default_rng(9)
    M, N, K = 6, 4, 5
    A = rnd(rng, *((M, K) if ta == ref.NoTrans else (K, M)))
    B = rnd(rng, *((K, N) if tb == ref.NoTrans else (N, K)))
    C = rnd(rng, M, N)
    c1, c2 = store(C, ref.ColMajor), store(C, ref.ColMajor)
    ref.gemm(ref.ColMajor, ta, tb, 0.7, store(A, ref.ColMajor), store(B, ref.ColMajor), 0.2, c1)
    Am = A if ta == ref.NoTrans else A.T.copy()
    Bm = B if tb == ref.NoTrans else B.T.copy()
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 0.7, store(Am, ref.ColMajor), store(Bm, ref.ColMajor), 0.2, c2)
    assert np.array_equal(np.asarray(c1), np.asarray(c2))
    # row-major storage of the same logical problem gives the same numbers
    c3 = store(C, ref.RowMajor, 2)
    ref.gemm(ref.RowMajor, ta, tb, 0.7, store(A, ref.RowMajor, 1), store(B, ref.RowMajor), 0.2, c3)
    assert np.array_equal(np.asarray(c1), np.asarray(c3))


# ---------------------------------------------------------------- SYRK ----

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_syrk_exact_and_other_triangle_untouched(order, uplo, trans):
    rng = np.random.default_rng(20 + uplo + trans)
    N, K = 6, 4
    A = rnd(rng, *((N, K) if trans == ref.NoTrans else (K, N)))
    C = rnd(rng, N, N)
    sentinel = 12345.678
    Cin = C.copy()
    for i in range(N):
        for j in range(N):
            if (uplo == ref.Lower and i < j) or (uplo == ref.Upper and i > j):
                Cin[i, j] = sentinel
    alpha, beta = -0.6, 0.9
    Cs = store(Cin, order, 2)
    ref.syrk(order, uplo, trans, alpha, store(A, order, 1), beta, Cs)
    Ae = exact.frac(A) if trans == ref.NoTrans else exact.transpose(exact.frac(A))
    P, Pabs = exact.matmul(Ae, exact.transpose(Ae)), exact.abs_matmul(Ae, exact.transpose(Ae))
    for i in range(N):
        for j in range(N):
            inside = (i >= j) if uplo == ref.Lower else (i <= j)
            if not inside:
                assert Cs[i, j] == sentinel
                continue
            want = Fraction(alpha) * P[i][j] + Fraction(beta) * Fraction(float(C[i, j]))
            bound = (K + 4) * U * float(abs(Fraction(alpha)) * Pabs[i][j] + abs(beta * C[i, j]))
            assert abs(Fraction(float(Cs[i, j])) - want) <= bound


def test_syrk_matches_gemm_on_triangle_and_beta_zero_ignores_nan():
    rng = np.random.default_rng(21)
    N, K = 7, 9
    A = rnd(rng, N, K)
    Cg = np.zeros((N, N), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.5, store(A, ref.ColMajor), store(A, ref.ColMajor), 0.0, Cg)
    Cs = np.full((N, N), np.nan, order="F")
    ref.syrk(ref.ColMajor, ref.Lower, ref.NoTrans, 1.5, store(A, ref.ColMajor), 0.0, Cs)
    low = np.tril_indices(N)
    assert np.array_equal(Cs[low], Cg[low])
    assert np.all(np.isnan(Cs[np.triu_indices(N, 1)]))


# ---------------------------------------------------------------- TRMM ----

FLAGS = list(itertools.product([ref.Left, ref.Right], [ref.Upper, ref.Lower], TRANS, [ref.NonUnit, ref.Unit]))


def poisoned_triangular(rng, n, uplo, diag):
    """Random matrix whose not-to-be-read entries are NaN."""
    A = rnd(rng, n, n) + np.diag(np.full(n, 3.0))
    P = A.copy()
    for r in range(n):
        for c in range(n):
            outside = (r < c) if uplo == ref.Lower else (r > c)
            if outside or (r == c and diag == ref.Unit):
                P[r, c] = np.nan
    return A, P


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_trmm_exact_rational_with_poison(order, side, uplo, trans, diag):
    rng = np.random.default_rng(side + 3 * uplo + 5 * trans + 7 * diag + order)
    M, N = 5, 4
    n = M if side == ref.Left else N
    A, P = poisoned_triangular(rng, n, uplo, diag)
    B = rnd(rng, M, N)
    alpha = 0.8
    Bs = store(B, order, 1)
    ref.trmm(order, side, uplo, trans, diag, alpha, store(P, order, 2), Bs)
    Tm = exact.triangle(exact.frac(A), uplo == ref.Lower, diag == ref.Unit)
    if trans == ref.Trans:
        Tm = exact.transpose(Tm)
    Be = exact.frac(B)
    W = exact.matmul(Tm, Be) if side == ref.Left else exact.matmul(Be, Tm)
    Wabs = exact.abs_matmul(Tm, Be) if side == ref.Left else exact.abs_matmul(Be, Tm)
    for i in range(M):
        for j in range(N):
            want = Fraction(alpha) * W[i][j]
            assert abs(Fraction(float(Bs[i, j])) - want) <= (n + 4) * U * float(Wabs[i][j]), (i, j)


def test_trmm_equals_gemm_with_explicit_triangle():
    rng = np.random.default_rng(31)
    M, N = 8, 6
    A = rnd(rng, M, M)
    B = rnd(rng, M, N)
    Bs = store(B, ref.ColMajor)
    ref.trmm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, 1.0, store(A, ref.ColMajor), Bs)
    Cg = np.zeros((M, N), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, store(np.tril(A), ref.ColMajor), store(B, ref.ColMajor), 0.0, Cg)
    assert np.max(np.abs(np.asarray(Bs) - Cg)) <= 16 * U * np.max(np.abs(Cg))


# ---------------------------------------------------------------- TRSM ----

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_trsm_exact_rational_with_poison(order, side, uplo, trans, diag):
    rng = np.random.default_rng(100 + side + 3 * uplo + 5 * trans + 7 * diag + order)
    M, N = 5, 4
    n = M if side == ref.Left else N
    A, P = poisoned_triangular(rng, n, uplo, diag)
    B = rnd(rng, M, N)
    alpha = -1.5
    Bs = store(B, order, 2)
    ref.trsm(order, side, uplo, trans, diag, alpha, store(P, order, 1), Bs)
    Tm = exact.triangle(exact.frac(A), uplo == ref.Lower, diag == ref.Unit)
    if trans == ref.Trans:
        Tm = exact.transpose(Tm)
    aB = [[Fraction(alpha) * v for v in row] for row in exact.frac(B)]
    if side == ref.Left:
        X = exact.solve_triangular(Tm, aB)
    else:   # X T = aB  <=>  T^T X^T = aB^T
        X = exact.transpose(exact.solve_triangular(exact.transpose(Tm), exact.transpose(aB)))
    got = np.asarray(Bs)
    want = exact.to_float(X)
    # diagonally shifted (3 + u) triangle of order 5: condition number is small
    assert np.max(np.abs(got - want)) <= 200 * U * np.max(np.abs(want))


@pytest.mark.parametrize("side,uplo,trans", list(itertools.product([ref.Left, ref.Right], [ref.Upper, ref.Lower], TRANS)))
def test_trsm_recovers_known_integer_solution_exactly(side, uplo, trans):
    """Unit-triangular integer A, integer X: B = op(A) X is exact and substitution stays in integers."""
    M, N = 9, 7
    n = M if side == ref.Left else N
    A = np.asarray(synth.matrix(n, n, seed=40, mat=0, integers=True))
    X = np.asarray(synth.matrix(M, N, seed=40, mat=1, integers=True))
    Tm = np.tril(A, -1) + np.eye(n) if uplo == ref.Lower else np.triu(A, 1) + np.eye(n)
    Tm = Tm if trans == ref.NoTrans else Tm.T
    B = Tm @ X if side == ref.Left else X @ Tm
    Bs = store(B / 2.0, ref.ColMajor, 1)          # alpha = 2 undoes the halving exactly
    ref.trsm(ref.ColMajor, side, uplo, trans, ref.Unit, 2.0, store(A, ref.ColMajor), Bs)
    assert np.array_equal(np.asarray(Bs), X)


def test_trsm_diagonal_and_identity_closed_forms():
    rng = np.random.default_rng(41)
    M, N = 6, 5
    d = rng.uniform(1, 2, M)
    B = rnd(rng, M, N)
    Bs = store(B, ref.ColMajor)
    ref.trsm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, 0.5, store(np.diag(d), ref.ColMajor), Bs)
    assert np.array_equal(np.asarray(Bs), (0.5 * B) / d[:, None])
    Bs = store(B, ref.ColMajor)
    Z = np.full((N, N), np.nan, order="F")        # unit diagonal, zero strict upper part, rest never read
    Z[np.triu_indices(N, 1)] = 0.0
    ref.trsm(ref.ColMajor, ref.Right, ref.Upper, ref.Trans, ref.Unit, 4.0, Z, Bs)
    assert np.array_equal(np.asarray(Bs), 4.0 * B)
    # alpha = 0: X = 0 and A is not read
    Bs = store(B, ref.ColMajor)
    ref.trsm(ref.ColMajor, ref.Left, ref.Upper, ref.NoTrans, ref.NonUnit, 0.0, np.full((M, M), np.nan, order="F"), Bs)
    assert np.array_equal(np.asarray(Bs), np.zeros((M, N)))


def test_trsm_then_trmm_roundtrip_dominant_triangle():
    """The benchmark's triangular workload: residual of the solve is at rounding level."""
    n, m = 96, 17
    A = synth.matrix(n, n, seed=42, mat=0)
    synth.dominant_diag(A, seed=42, mat=0)
    B = synth.matrix(n, m, seed=42, mat=1)
    X = B.copy(order="F")
    ref.trsm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, 1.0, A, X)
    R = X.copy(order="F")
    ref.trmm(ref.ColMajor, ref.Left, ref.Lower, ref.NoTrans, ref.NonUnit, 1.0, A, R)
    res = np.linalg.norm(R - B) / (np.linalg.norm(np.tril(A)) * np.linalg.norm(X))
    assert res < 1e-15


# ------------------------------------------------------------- generator --

def test_generator_is_element_addressable_and_in_range():
    A = synth.matrix(37, 11, seed=0, mat=0, ld=40)
    assert A.min() >= -1.0 and A.max() < 1.0
    for (i, j) in [(0, 0), (36, 10), (5, 3)]:
        assert A[i, j] == synth.element(0, 0, i, j, 37)
    assert abs(float(np.mean(synth.matrix(400, 400, seed=1, mat=1)))) < 0.01
    Af = synth.matrix(37, 11, seed=0, mat=0, dtype=np.float32)
    assert np.array_equal(Af, A.astype(np.float32))
    assert not np.array_equal(synth.matrix(8, 8, 0, 0), synth.matrix(8, 8, 0, 1))
    assert not np.array_equal(synth.matrix(8, 8, 0, 0), synth.matrix(8, 8, 1, 0))


# ------------------------------------------------------- SYR2K / SYMM -----

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_syr2k_exact_and_other_triangle_untouched(order, uplo, trans):
    rng = np.random.default_rng(50 + uplo + trans + order)
    N, K = 6, 4
    shape = (N, K) if trans == ref.NoTrans else (K, N)
    A, B = rnd(rng, *shape), rnd(rng, *shape)
    C = rnd(rng, N, N)
    Cin = C.copy()
    outside = [(i, j) for i in range(N) for j in range(N) if ((i < j) if uplo == ref.Lower else (i > j))]
    for (i, j) in outside:
        Cin[i, j] = -999.25
    alpha, beta = 0.7, -0.4
    Cs = store(Cin, order, 1)
    ref.syr2k(order, uplo, trans, alpha, store(A, order, 2), store(B, order), beta, Cs)
    Ae = exact.frac(A) if trans == ref.NoTrans else exact.transpose(exact.frac(A))
    Be = exact.frac(B) if trans == ref.NoTrans else exact.transpose(exact.frac(B))
    P1, P2 = exact.matmul(Ae, exact.transpose(Be)), exact.matmul(Be, exact.transpose(Ae))
    Q = exact.abs_matmul(Ae, exact.transpose(Be))
    for i in range(N):
        for j in range(N):
            if (i, j) in outside:
                assert Cs[i, j] == -999.25
                continue
            want = Fraction(alpha) * (P1[i][j] + P2[i][j]) + Fraction(beta) * Fraction(float(C[i, j]))
            bound = (2 * K + 6) * U * float(2 * abs(Fraction(alpha)) * Q[i][j] + abs(beta * C[i, j])) + 1e-300
            assert abs(Fraction(float(Cs[i, j])) - want) <= bound + 4 * U * float(abs(want))


def test_syr2k_with_b_equal_a_is_twice_syrk_and_result_is_symmetric():
    N, K = 7, 5
    A = np.asarray(synth.matrix(N, K, 51, 0, integers=True))
    B = np.asarray(synth.matrix(N, K, 51, 1, integers=True))
    C2 = np.zeros((N, N), order="F")
    ref.syr2k(ref.ColMajor, ref.Lower, ref.NoTrans, 1.0, store(A, ref.ColMajor), store(A, ref.ColMajor), 0.0, C2)
    C1 = np.zeros((N, N), order="F")
    ref.syrk(ref.ColMajor, ref.Lower, ref.NoTrans, 2.0, store(A, ref.ColMajor), 0.0, C1)
    assert np.array_equal(np.tril(C2), np.tril(C1))
    lo, up = np.zeros((N, N), order="F"), np.zeros((N, N), order="F")
    ref.syr2k(ref.ColMajor, ref.Lower, ref.NoTrans, 1.0, store(A, ref.ColMajor), store(B, ref.ColMajor), 0.0, lo)
    ref.syr2k(ref.ColMajor, ref.Upper, ref.NoTrans, 1.0, store(A, ref.ColMajor), store(B, ref.ColMajor), 0.0, up)
    assert np.array_equal(np.tril(lo), np.triu(up).T)
    assert np.array_equal(np.tril(lo), np.tril(A @ B.T + B @ A.T))        # integers: exact


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side", [ref.Left, ref.Right])
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
def test_symm_exact_with_poisoned_other_triangle(order, side, uplo):
    rng = np.random.default_rng(60 + side + uplo + order)
    M, N = 5, 4
    n = M if side == ref.Left else N
    S = rnd(rng, n, n)
    S = (S + S.T) / 2.0                       # the symmetric matrix the stored triangle stands for
    P = S.copy()
    for r in range(n):
        for c in range(n):
            if (r < c) if uplo == ref.Lower else (r > c):
                P[r, c] = np.nan                # never read
    B, C = rnd(rng, M, N), rnd(rng, M, N)
    alpha, beta = -1.1, 0.6
    Cs = store(C, order, 2)
    ref.symm(order, side, uplo, alpha, store(P, order, 1), store(B, order), beta, Cs)
    Se, Be = exact.frac(S), exact.frac(B)
    W = exact.matmul(Se, Be) if side == ref.Left else exact.matmul(Be, Se)
    Wabs = exact.abs_matmul(Se, Be) if side == ref.Left else exact.abs_matmul(Be, Se)
    for i in range(M):
        for j in range(N):
            want = Fraction(alpha) * W[i][j] + Fraction(beta) * Fraction(float(C[i, j]))
            bound = (n + 4) * U * float(abs(Fraction(alpha)) * Wabs[i][j] + abs(beta * C[i, j]))
            assert abs(Fraction(float(Cs[i, j])) - want) <= bound, (i, j)


def test_symm_equals_gemm_with_the_full_symmetric_matrix():
    M, N = 9, 6
    S = np.asarray(synth.matrix(M, M, 61, 0, integers=True))
    S = np.tril(S) + np.tril(S, -1).T
    B = np.asarray(synth.matrix(M, N, 61, 1, integers=True))
    Cg = np.zeros((M, N), order="F")
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, store(S, ref.ColMajor), store(B, ref.ColMajor), 0.0, Cg)
    Cs = np.zeros((M, N), order="F")
    ref.symm(ref.ColMajor, ref.Left, ref.Lower, 1.0, store(np.tril(S) + np.triu(np.full((M, M), 77.0), 1), ref.ColMajor),
             store(B, ref.ColMajor), 0.0, Cs)
    assert np.array_equal(Cs, Cg)


# ------------------------------------------- single-precision entry points -----
# ref_ssyrk / ref_ssyr2k / ref_ssymm / ref_strmm / ref_strsm are instantiations of the bodies
# pinned above with float storage: they read float32, accumulate in double and round once.  Each is
# pinned on its own (exact rationals with a one-rounding bound, integers bit-exact, NaN on everything
# that must not be read), through the same binding the GPU parity tests use.

U32 = 2.0 ** -24


def one_rounding(got, want, slack=0.0):
    """|got - want| within one float32 rounding of a double-precision result of relative error `slack`."""
    want = float(want)
    return abs(float(got) - want) <= (U32 * 1.0001 + slack) * abs(want) + 1e-37


def f32(a):
    return np.asarray(a, dtype=np.float32)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_ssyrk_one_rounding_and_other_triangle_untouched(order, uplo, trans):
    rng = np.random.default_rng(70 + uplo + trans + order)
    N, K = 5, 40
    A = f32(rnd(rng, *((N, K) if trans == ref.NoTrans else (K, N))))
    C = f32(rnd(rng, N, N))
    Cin = C.copy()
    outside = [(i, j) for i in range(N) for j in range(N) if ((i < j) if uplo == ref.Lower else (i > j))]
    for (i, j) in outside:
        Cin[i, j] = np.float32(-777.5)
    alpha, beta = 0.75, -0.5
    Cs = store(Cin, order, 2, dtype=np.float32)
    ref.syrk(order, uplo, trans, alpha, store(A, order, 1, dtype=np.float32), beta, Cs)
    assert Cs.dtype == np.float32
    Ae = exact.frac(A) if trans == ref.NoTrans else exact.transpose(exact.frac(A))
    P = exact.matmul(Ae, exact.transpose(Ae))
    for i in range(N):
        for j in range(N):
            if (i, j) in outside:
                assert Cs[i, j] == np.float32(-777.5)
                continue
            want = Fraction(alpha) * P[i][j] + Fraction(beta) * Fraction(float(C[i, j]))
            assert one_rounding(Cs[i, j], want, (K + 4) * U * 8), (i, j)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
@pytest.mark.parametrize("trans", TRANS)
def test_ssyr2k_one_rounding_integers_exact_and_other_triangle_untouched(order, uplo, trans):
    rng = np.random.default_rng(80 + uplo + trans + order)
    N, K = 6, 30
    shape = (N, K) if trans == ref.NoTrans else (K, N)
    A, B = f32(rnd(rng, *shape)), f32(rnd(rng, *shape))
    Cin = np.full((N, N), np.nan, dtype=np.float32)        # beta = 0: nothing of C is read
    Cs = store(Cin, order, 1, dtype=np.float32)
    ref.syr2k(order, uplo, trans, -1.25, store(A, order, 2, dtype=np.float32), store(B, order, dtype=np.float32), 0.0, Cs)
    Ae = exact.frac(A) if trans == ref.NoTrans else exact.transpose(exact.frac(A))
    Be = exact.frac(B) if trans == ref.NoTrans else exact.transpose(exact.frac(B))
    P1, P2 = exact.matmul(Ae, exact.transpose(Be)), exact.matmul(Be, exact.transpose(Ae))
    Q = exact.abs_matmul(Ae, exact.transpose(Be))
    for i in range(N):
        for j in range(N):
            inside = (i >= j) if uplo == ref.Lower else (i <= j)
            if not inside:
                assert np.isnan(Cs[i, j])
                continue
            want = Fraction(-1.25) * (P1[i][j] + P2[i][j])
            err = abs(Fraction(float(Cs[i, j])) - want)
            assert err <= U32 * 1.0001 * abs(want) + (2 * K + 6) * U * float(2 * 1.25 * Q[i][j]), (i, j)
    # small integers: every product and sum is exact, also after the rounding to float32
    Ai = f32(np.asarray(synth.matrix(N, K, 81, 0, integers=True)))
    Bi = f32(np.asarray(synth.matrix(N, K, 81, 1, integers=True)))
    Ci = np.zeros((N, N), dtype=np.float32, order="F")
    ref.syr2k(ref.ColMajor, uplo, ref.NoTrans, 1.0, store(Ai, ref.ColMajor, dtype=np.float32), store(Bi, ref.ColMajor, dtype=np.float32), 0.0, Ci)
    full = Ai.astype(np.float64) @ Bi.astype(np.float64).T + Bi.astype(np.float64) @ Ai.astype(np.float64).T
    tri = np.tril if uplo == ref.Lower else np.triu
    assert np.array_equal(tri(Ci).astype(np.float64), tri(full))


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side", [ref.Left, ref.Right])
@pytest.mark.parametrize("uplo", [ref.Upper, ref.Lower])
def test_ssymm_one_rounding_with_poisoned_other_triangle(order, side, uplo):
    rng = np.random.default_rng(90 + side + uplo + order)
    M, N = 6, 5
    n = M if side == ref.Left else N
    S = f32(rnd(rng, n, n))
    S = np.tril(S) + np.tril(S, -1).T                     # symmetric, exactly representable
    P = S.copy()
    for r in range(n):
        for c in range(n):
            if (r < c) if uplo == ref.Lower else (r > c):
                P[r, c] = np.nan
    B, C = f32(rnd(rng, M, N)), f32(rnd(rng, M, N))
    alpha, beta = 1.5, 0.25
    Cs = store(C, order, 2, dtype=np.float32)
    ref.symm(order, side, uplo, alpha, store(P, order, 1, dtype=np.float32), store(B, order, dtype=np.float32), beta, Cs)
    Se, Be = exact.frac(S), exact.frac(B)
    W = exact.matmul(Se, Be) if side == ref.Left else exact.matmul(Be, Se)
    Wabs = exact.abs_matmul(Se, Be) if side == ref.Left else exact.abs_matmul(Be, Se)
    for i in range(M):
        for j in range(N):
            want = Fraction(alpha) * W[i][j] + Fraction(beta) * Fraction(float(C[i, j]))
            err = abs(Fraction(float(Cs[i, j])) - want)
            assert err <= U32 * 1.0001 * abs(want) + (n + 4) * U * float(alpha * Wabs[i][j] + abs(beta * C[i, j])), (i, j)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_strmm_one_rounding_with_poison(order, side, uplo, trans, diag):
    rng = np.random.default_rng(110 + side + 3 * uplo + 5 * trans + 7 * diag + order)
    M, N = 5, 6
    n = M if side == ref.Left else N
    A, P = poisoned_triangular(rng, n, uplo, diag)
    A, P = f32(A), f32(P)
    B = f32(rnd(rng, M, N))
    alpha = -0.75
    Bs = store(B, order, 1, dtype=np.float32)
    ref.trmm(order, side, uplo, trans, diag, alpha, store(P, order, 2, dtype=np.float32), Bs)
    Tm = exact.triangle(exact.frac(A), uplo == ref.Lower, diag == ref.Unit)
    if trans == ref.Trans:
        Tm = exact.transpose(Tm)
    Be = exact.frac(B)
    W = exact.matmul(Tm, Be) if side == ref.Left else exact.matmul(Be, Tm)
    Wabs = exact.abs_matmul(Tm, Be) if side == ref.Left else exact.abs_matmul(Be, Tm)
    for i in range(M):
        for j in range(N):
            want = Fraction(alpha) * W[i][j]
            err = abs(Fraction(float(Bs[i, j])) - want)
            assert err <= U32 * 1.0001 * abs(want) + (n + 4) * U * float(Wabs[i][j]), (i, j)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_strsm_one_rounding_with_poison(order, side, uplo, trans, diag):
    rng = np.random.default_rng(130 + side + 3 * uplo + 5 * trans + 7 * diag + order)
    M, N = 5, 4
    n = M if side == ref.Left else N
    A, P = poisoned_triangular(rng, n, uplo, diag)
    A, P = f32(A), f32(P)
    B = f32(rnd(rng, M, N))
    alpha = 2.5
    Bs = store(B, order, 2, dtype=np.float32)
    ref.trsm(order, side, uplo, trans, diag, alpha, store(P, order, 1, dtype=np.float32), Bs)
    Tm = exact.triangle(exact.frac(A), uplo == ref.Lower, diag == ref.Unit)
    if trans == ref.Trans:
        Tm = exact.transpose(Tm)
    aB = [[Fraction(alpha) * v for v in row] for row in exact.frac(B)]
    if side == ref.Left:
        X = exact.solve_triangular(Tm, aB)
    else:
        X = exact.transpose(exact.solve_triangular(exact.transpose(Tm), exact.transpose(aB)))
    got, want = np.asarray(Bs, dtype=np.float64), exact.to_float(X)
    assert Bs.dtype == np.float32 and np.all(np.isfinite(got))
    # the substitution runs in double (error as in the double-precision pin), then one float32 rounding
    assert np.all(np.abs(got - want) <= U32 * 1.0001 * np.abs(want) + 200 * U * np.max(np.abs(want)))


@pytest.mark.parametrize("side,uplo,trans", list(itertools.product([ref.Left, ref.Right], [ref.Upper, ref.Lower], TRANS)))
def test_strsm_recovers_known_integer_solution_and_strmm_forms_it_exactly(side, uplo, trans):
    rng = np.random.default_rng(150 + side + uplo + trans)
    M, N = 7, 6
    n = M if side == ref.Left else N
    L = np.tril(rng.integers(-2, 3, (n, n)), -1) + np.diag(rng.choice([1, 2, 4], n))      # powers of two divide exactly
    Tm = (L if uplo == ref.Lower else L.T).astype(np.float32)
    X = rng.integers(-3, 4, (M, N)).astype(np.float32)
    op = Tm.T if trans == ref.Trans else Tm
    Bv = (op.astype(np.float64) @ X if side == ref.Left else X @ op.astype(np.float64)).astype(np.float32)
    Bt = store(X, ref.ColMajor, dtype=np.float32)
    ref.trmm(ref.ColMajor, side, uplo, trans, ref.NonUnit, 1.0, store(Tm, ref.ColMajor, dtype=np.float32), Bt)
    assert np.array_equal(np.asarray(Bt), Bv)
    Bs = store(Bv, ref.ColMajor, 1, dtype=np.float32)
    ref.trsm(ref.ColMajor, side, uplo, trans, ref.NonUnit, 1.0, store(Tm, ref.ColMajor, dtype=np.float32), Bs)
    assert np.array_equal(np.asarray(Bs), X)


def test_single_precision_entry_points_agree_with_double_ones_rounded_once():
    """Inputs that float32 holds exactly: the s-function must return the d-function's result rounded."""
    rng = np.random.default_rng(170)
    N, K = 9, 11
    A32, B32, C32 = f32(rnd(rng, N, K)), f32(rnd(rng, N, K)), f32(rnd(rng, N, N))
    A64, B64, C64 = A32.astype(np.float64), B32.astype(np.float64), C32.astype(np.float64)
    F = lambda a, dt: store(a, ref.ColMajor, dtype=dt)
    for uplo in (ref.Upper, ref.Lower):
        tri = np.tril if uplo == ref.Lower else np.triu
        cs, cd = F(C32, np.float32), F(C64, np.float64)
        ref.syrk(ref.ColMajor, uplo, ref.NoTrans, 0.3, F(A32, np.float32), 1.7, cs)
        ref.syrk(ref.ColMajor, uplo, ref.NoTrans, 0.3, F(A64, np.float64), 1.7, cd)
        assert np.array_equal(tri(np.asarray(cs)), tri(np.asarray(cd).astype(np.float32)))
        cs, cd = F(C32, np.float32), F(C64, np.float64)
        ref.syr2k(ref.ColMajor, uplo, ref.NoTrans, 0.3, F(A32, np.float32), F(B32, np.float32), 1.7, cs)
        ref.syr2k(ref.ColMajor, uplo, ref.NoTrans, 0.3, F(A64, np.float64), F(B64, np.float64), 1.7, cd)
        assert np.array_equal(tri(np.asarray(cs)), tri(np.asarray(cd).astype(np.float32)))
        S32 = f32(rnd(rng, N, N))
        bs, bd = F(A32, np.float32), F(A64, np.float64)
        ref.symm(ref.ColMajor, ref.Left, uplo, 1.0, F(S32, np.float32), F(B32, np.float32), 0.0, bs)
        ref.symm(ref.ColMajor, ref.Left, uplo, 1.0, F(S32.astype(np.float64), np.float64), F(B64, np.float64), 0.0, bd)
        assert np.array_equal(np.asarray(bs), np.asarray(bd).astype(np.float32))
        T32 = S32 + np.diag(np.full(N, 4.0, dtype=np.float32))
        for fn in (ref.trmm, ref.trsm):
            bs, bd = F(B32, np.float32), F(B64, np.float64)
            fn(ref.ColMajor, ref.Left, uplo, ref.Trans, ref.NonUnit, 0.5, F(T32, np.float32), bs)
            fn(ref.ColMajor, ref.Left, uplo, ref.Trans, ref.NonUnit, 0.5, F(T32.astype(np.float64), np.float64), bd)
            assert np.array_equal(np.asarray(bs), np.asarray(bd).astype(np.float32))
