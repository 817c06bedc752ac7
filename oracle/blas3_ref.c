/*
 * ORACLE -- test infrastructure only.
 *
 * Plain, slow, un-tiled CPU definitions of the level-3 BLAS routines that the
 * tile algorithms of the paper (Section III.B, Eq. 1a-1f) must reproduce.  The
 * tile method is exact up to the order of floating-point summation, so the
 * oracle is the textbook definition of each routine written out as loops over
 * whole matrices: no tiling, no blocking, no reordering beyond "sum over l in
 * increasing order".  Nothing here is shared with, or included by, the GPU
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.
 *
 * Conventions (the BLAS standard that Section II of the paper refers to):
 *   order  101 row-major, 102 column-major
 *   trans  111 no-transpose, 112 transpose, 113 conjugate-transpose (= 112, real)
 *   uplo   121 upper, 122 lower
 *   diag   131 non-unit, 132 unit
 *   side   141 left, 142 right
 * Element (r,c) of a matrix with leading dimension ld is x[r + c*ld] in
 * column-major order and x[r*ld + c] in row-major order.
 *
 * Readings where the paper is silent or at odds with the standard:
 *   - Eq. 1c (TRSM) and Eq. 1d (TRMM) are printed with alpha in places that do
 *     not match the standard once applied to every tile; the standard is
 *     followed: TRSM solves op(A) X = alpha B (or X op(A) = alpha B), TRMM
 *     forms alpha op(A) B (or alpha B op(A)).
 *   - beta == 0 means C is not read (NaN/Inf in C do not propagate);
 *     alpha == 0 means A and B are not read.
 *   - The triangular routines read only the named triangle of A, and with a
 *     unit diagonal do not read the diagonal either.
 *   - Single precision inputs are accumulated in double and rounded once.
 *
 * Every function returns 0, or -(k) when its k-th argument is invalid.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

enum { ROW = 101, COL = 102, NOTR = 111, TR = 112, CTR = 113,
       UP = 121, LO = 122, NONUNIT = 131, UNIT = 132, LEFT = 141, RIGHT = 142 };

static inline size_t at(int order, long r, long c, long ld)
{
    return order == COL ? (size_t)r + (size_t)c * (size_t)ld
                        : (size_t)r * (size_t)ld + (size_t)c;
}

static inline int is_tr(int t) { return t == TR || t == CTR; }

/* ------------------------------------------------------------------ GEMM --
 * C(i,j) <- alpha * sum_{l<K} op(A)(i,l) * op(B)(l,j) + beta * C(i,j)
 * (Eq. 1a with a single tile).  For each output column the sums for all rows
 * are advanced together, l increasing.
 */
#define DEFINE_GEMM(NAME, T)                                                        \
int NAME(int order, int ta, int tb, int M, int N, int K, double alpha,              \
         const T *A, int lda, const T *B, int ldb, double beta, T *C, int ldc)      \
{                                                                                   \
    if (order != ROW && order != COL) return -1;                                    \
    if (ta != NOTR && !is_tr(ta)) return -2;                                        \
    if (tb != NOTR && !is_tr(tb)) return -3;                                        \
    if (M < 0) return -4;                                                           \
    if (N < 0) return -5;                                                           \
    if (K < 0) return -6;                                                           \
    if (M == 0 || N == 0) return 0;                                                 \
    int bad = 0;                                                                    \
    _Pragma("omp parallel for schedule(dynamic, 1) reduction(|:bad)")               \
    for (long j = 0; j < N; ++j) {                                                  \
        double *acc = (double *)calloc((size_t)M, sizeof(double));                  \
        if (!acc) { bad |= 1; continue; }                                           \
        if (alpha != 0.0) {                                                         \
            for (long l = 0; l < K; ++l) {                                          \
                double b = is_tr(tb) ? (double)B[at(order, j, l, ldb)]              \
                                     : (double)B[at(order, l, j, ldb)];             \
                for (long i = 0; i < M; ++i) {                                      \
                    double a = is_tr(ta) ? (double)A[at(order, l, i, lda)]          \
                                         : (double)A[at(order, i, l, lda)];         \
                    acc[i] += a * b;                                                \
                }                                                                   \
            }                                                                       \
        }                                                                           \
        for (long i = 0; i < M; ++i) {                                              \
            size_t p = at(order, i, j, ldc);                                        \
            double v = (alpha != 0.0) ? alpha * acc[i] : 0.0;                       \
            if (beta != 0.0) v += beta * (double)C[p];                              \
            C[p] = (T)v;                                                            \
        }                                                                           \
        free(acc);                                                                  \
    }                                                                               \
    return bad ? 100 : 0;                                                           \
}

DEFINE_GEMM(ref_dgemm, double)
DEFINE_GEMM(ref_sgemm, float)

/* ------------------------------------------------------------------ SYRK --
 * trans = N:  C <- alpha * A * A^T + beta * C,  A is N x K
 * trans = T:  C <- alpha * A^T * A + beta * C,  A is K x N
 * Only the uplo triangle of C (diagonal included) is read or written
 * (Eq. 1b with a single tile).
 */
#define DEFINE_SYRK(NAME, T)                                                        \
int NAME(int order, int uplo, int trans, int N, int K, double alpha,                \
         const T *A, int lda, double beta, T *C, int ldc)                           \
{                                                                                   \
    if (order != ROW && order != COL) return -1;                                    \
    if (uplo != UP && uplo != LO) return -2;                                        \
    if (trans != NOTR && !is_tr(trans)) return -3;                                  \
    if (N < 0) return -4;                                                           \
    if (K < 0) return -5;                                                           \
    _Pragma("omp parallel for schedule(dynamic, 1)")                                \
    for (long j = 0; j < N; ++j) {                                                  \
        long i0 = (uplo == LO) ? j : 0;                                             \
        long i1 = (uplo == LO) ? N : j + 1;                                         \
        for (long i = i0; i < i1; ++i) {                                            \
            double s = 0.0;                                                         \
            if (alpha != 0.0)                                                       \
                for (long l = 0; l < K; ++l) {                                      \
                    double x = is_tr(trans) ? (double)A[at(order, l, i, lda)]       \
                                            : (double)A[at(order, i, l, lda)];      \
                    double y = is_tr(trans) ? (double)A[at(order, l, j, lda)]       \
                                            : (double)A[at(order, j, l, lda)];      \
                    s += x * y;                                                     \
                }                                                                   \
            size_t p = at(order, i, j, ldc);                                        \
            double v = (alpha != 0.0) ? alpha * s : 0.0;                            \
            if (beta != 0.0) v += beta * (double)C[p];                              \
            C[p] = (T)v;                                                            \
        }                                                                           \
    }                                                                               \
    return 0;                                                                       \
}

DEFINE_SYRK(ref_dsyrk, double)
DEFINE_SYRK(ref_ssyrk, float)

/* ----------------------------------------------------------------- SYR2K --
 * trans = N:  C <- alpha * (A * B^T + B * A^T) + beta * C,  A and B are N x K
 * trans = T:  C <- alpha * (A^T * B + B^T * A) + beta * C,  A and B are K x N
 * Only the uplo triangle of C is read or written (Eq. 1e with a single tile).
 */
#define DEFINE_SYR2K(NAME, T)                                                       \
int NAME(int order, int uplo, int trans, int N, int K, double alpha,                \
         const T *A, int lda, const T *B, int ldb, double beta, T *C, int ldc)      \
{                                                                                   \
    if (order != ROW && order != COL) return -1;                                    \
    if (uplo != UP && uplo != LO) return -2;                                        \
    if (trans != NOTR && !is_tr(trans)) return -3;                                  \
    if (N < 0) return -4;                                                           \
    if (K < 0) return -5;                                                           \
    _Pragma("omp parallel for schedule(dynamic, 1)")                                \
    for (long j = 0; j < N; ++j) {                                                  \
        long i0 = (uplo == LO) ? j : 0;                                             \
        long i1 = (uplo == LO) ? N : j + 1;                                         \
        for (long i = i0; i < i1; ++i) {                                            \
            double s = 0.0;                                                         \
            if (alpha != 0.0)                                                       \
                for (long l = 0; l < K; ++l) {                                      \
                    double ai = is_tr(trans) ? (double)A[at(order, l, i, lda)] : (double)A[at(order, i, l, lda)]; \
                    double aj = is_tr(trans) ? (double)A[at(order, l, j, lda)] : (double)A[at(order, j, l, lda)]; \
                    double bi = is_tr(trans) ? (double)B[at(order, l, i, ldb)] : (double)B[at(order, i, l, ldb)]; \
                    double bj = is_tr(trans) ? (double)B[at(order, l, j, ldb)] : (double)B[at(order, j, l, ldb)]; \
                    s += ai * bj + bi * aj;                                         \
                }                                                                   \
            size_t p = at(order, i, j, ldc);                                        \
            double v = (alpha != 0.0) ? alpha * s : 0.0;                            \
            if (beta != 0.0) v += beta * (double)C[p];                              \
            C[p] = (T)v;                                                            \
        }                                                                           \
    }                                                                               \
    return 0;                                                                       \
}

DEFINE_SYR2K(ref_dsyr2k, double)
DEFINE_SYR2K(ref_ssyr2k, float)

/* ------------------------------------------------------------------ SYMM --
 * side = L:  C <- alpha * A * B + beta * C,  A is M x M symmetric
 * side = R:  C <- alpha * B * A + beta * C,  A is N x N symmetric
 * Only the uplo triangle of A (with its diagonal) is read; the rest of the
 * symmetric matrix is taken from it by reflection (Eq. 1f with a single tile).
 */
#define DEFINE_SYMM(NAME, T)                                                        \
int NAME(int order, int side, int uplo, int M, int N, double alpha,                 \
         const T *A, int lda, const T *B, int ldb, double beta, T *C, int ldc)      \
{                                                                                   \
    if (order != ROW && order != COL) return -1;                                    \
    if (side != LEFT && side != RIGHT) return -2;                                   \
    if (uplo != UP && uplo != LO) return -3;                                        \
    if (M < 0) return -4;                                                           \
    if (N < 0) return -5;                                                           \
    _Pragma("omp parallel for schedule(dynamic, 1)")                                \
    for (long j = 0; j < N; ++j) {                                                  \
        for (long i = 0; i < M; ++i) {                                              \
            double s = 0.0;                                                         \
            if (alpha != 0.0) {                                                     \
                long n = (side == LEFT) ? M : N;                                    \
                for (long l = 0; l < n; ++l) {                                      \
                    /* element (r, c) of the symmetric matrix */                    \
                    long r = (side == LEFT) ? i : l, c = (side == LEFT) ? l : j;    \
                    int stored = (uplo == LO) ? (r >= c) : (r <= c);                \
                    double a = stored ? (double)A[at(order, r, c, lda)] : (double)A[at(order, c, r, lda)]; \
                    double b = (side == LEFT) ? (double)B[at(order, l, j, ldb)] : (double)B[at(order, i, l, ldb)]; \
                    s += (side == LEFT) ? a * b : b * a;                            \
                }                                                                   \
            }                                                                       \
            size_t p = at(order, i, j, ldc);                                        \
            double v = (alpha != 0.0) ? alpha * s : 0.0;                            \
            if (beta != 0.0) v += beta * (double)C[p];                              \
            C[p] = (T)v;                                                            \
        }                                                                           \
    }                                                                               \
    return 0;                                                                       \
}

DEFINE_SYMM(ref_dsymm, double)
DEFINE_SYMM(ref_ssymm, float)

/* -------------------------------------------------- triangular operand ----
 * tri(r,c): the triangular matrix that A stands for -- the named triangle of
 * A, a diagonal of ones when diag is unit, zero elsewhere (never read there).
 * top(r,c): op(A) = tri or tri^T.
 */
#define DEFINE_TRI(T, SFX)                                                          \
static inline double tri_##SFX(int order, int uplo, int diag, const T *A, long lda, \
                               long r, long c)                                      \
{                                                                                   \
    if (r == c) return diag == UNIT ? 1.0 : (double)A[at(order, r, r, lda)];        \
    int inside = (uplo == LO) ? (r > c) : (r < c);                                  \
    return inside ? (double)A[at(order, r, c, lda)] : 0.0;                          \
}                                                                                   \
static inline double top_##SFX(int order, int uplo, int trans, int diag,            \
                               const T *A, long lda, long r, long c)                \
{                                                                                   \
    return is_tr(trans) ? tri_##SFX(order, uplo, diag, A, lda, c, r)                \
                        : tri_##SFX(order, uplo, diag, A, lda, r, c);               \
}

DEFINE_TRI(double, d)
DEFINE_TRI(float, s)

static int tri_args(int order, int side, int uplo, int trans, int diag, int M, int N)
{
    if (order != ROW && order != COL) return -1;
    if (side != LEFT && side != RIGHT) return -2;
    if (uplo != UP && uplo != LO) return -3;
    if (trans != NOTR && !is_tr(trans)) return -4;
    if (diag != UNIT && diag != NONUNIT) return -5;
    if (M < 0) return -6;
    if (N < 0) return -7;
    return 0;
}

/* ------------------------------------------------------------------ TRMM --
 * side = L:  B <- alpha * op(A) * B,  A is M x M
 * side = R:  B <- alpha * B * op(A),  A is N x N
 * Formed out of place from a copy of B, so no update order is implied
 * (Eq. 1d with a single tile, alpha on every term).
 */
#define DEFINE_TRMM(NAME, T, SFX)                                                   \
int NAME(int order, int side, int uplo, int trans, int diag, int M, int N,          \
         double alpha, const T *A, int lda, T *B, int ldb)                          \
{                                                                                   \
    int rc = tri_args(order, side, uplo, trans, diag, M, N);                        \
    if (rc) return rc;                                                              \
    if (M == 0 || N == 0) return 0;                                                 \
    double *old = (double *)malloc((size_t)M * (size_t)N * sizeof(double));         \
    if (!old) return 100;                                                           \
    for (long j = 0; j < N; ++j)                                                    \
        for (long i = 0; i < M; ++i)                                                \
            old[(size_t)i + (size_t)j * (size_t)M] = (double)B[at(order, i, j, ldb)]; \
    /* op(A) is lower triangular when exactly one of (uplo==lower, trans) holds */  \
    int eff_lower = (uplo == LO) != (is_tr(trans) != 0);                            \
    _Pragma("omp parallel for schedule(dynamic, 1)")                                \
    for (long j = 0; j < N; ++j) {                                                  \
        for (long i = 0; i < M; ++i) {                                              \
            double s = 0.0;                                                         \
            if (alpha != 0.0) {                                                     \
                if (side == LEFT) {                                                 \
                    long l0 = eff_lower ? 0 : i, l1 = eff_lower ? i + 1 : M;        \
                    for (long l = l0; l < l1; ++l)                                  \
                        s += top_##SFX(order, uplo, trans, diag, A, lda, i, l)      \
                             * old[(size_t)l + (size_t)j * (size_t)M];              \
                } else {                                                            \
                    long l0 = eff_lower ? j : 0, l1 = eff_lower ? N : j + 1;        \
                    for (long l = l0; l < l1; ++l)                                  \
                        s += old[(size_t)i + (size_t)l * (size_t)M]                 \
                             * top_##SFX(order, uplo, trans, diag, A, lda, l, j);   \
                }                                                                   \
            }                                                                       \
            B[at(order, i, j, ldb)] = (T)((alpha != 0.0) ? alpha * s : 0.0);        \
        }                                                                           \
    }                                                                               \
    free(old);                                                                      \
    return 0;                                                                       \
}

DEFINE_TRMM(ref_dtrmm, double, d)
DEFINE_TRMM(ref_strmm, float, s)

/* ------------------------------------------------------------------ TRSM --
 * side = L:  solve op(A) * X = alpha * B,  A is M x M
 * side = R:  solve X * op(A) = alpha * B,  A is N x N
 * X overwrites B.  Substitution, one unknown at a time (Eq. 1c with a single
 * tile, alpha applied to B only).
 *   left,  op(A) lower: x_i = (alpha b_i - sum_{l<i} op(A)(i,l) x_l) / op(A)(i,i), i up
 *   left,  op(A) upper: same with l>i, i down
 *   right: row i of X solves x op(A) = alpha b, i.e. column c uses
 *          x_c = (alpha b_c - sum_l x_l op(A)(l,c)) / op(A)(c,c),
 *          l<c (c up) when op(A) is upper, l>c (c down) when lower.
 */
#define DEFINE_TRSM(NAME, T, SFX)                                                   \
int NAME(int order, int side, int uplo, int trans, int diag, int M, int N,          \
         double alpha, const T *A, int lda, T *B, int ldb)                          \
{                                                                                   \
    int rc = tri_args(order, side, uplo, trans, diag, M, N);                        \
    if (rc) return rc;                                                              \
    if (M == 0 || N == 0) return 0;                                                 \
    if (alpha == 0.0) { /* X = 0 and A is not read */                               \
        for (long j = 0; j < N; ++j)                                                \
            for (long i = 0; i < M; ++i) B[at(order, i, j, ldb)] = (T)0;            \
        return 0;                                                                   \
    }                                                                               \
    int eff_lower = (uplo == LO) != (is_tr(trans) != 0);                            \
    if (side == LEFT) {                                                             \
        _Pragma("omp parallel for schedule(dynamic, 1)")                            \
        for (long j = 0; j < N; ++j) {                                              \
            double *x = (double *)malloc((size_t)M * sizeof(double));               \
            for (long t = 0; t < M; ++t) {                                          \
                long i = eff_lower ? t : M - 1 - t;                                 \
                double s = (alpha != 0.0) ? alpha * (double)B[at(order, i, j, ldb)] : 0.0; \
                long l0 = eff_lower ? 0 : i + 1, l1 = eff_lower ? i : M;            \
                for (long l = l0; l < l1; ++l)                                      \
                    s -= top_##SFX(order, uplo, trans, diag, A, lda, i, l) * x[l];  \
                x[i] = s / top_##SFX(order, uplo, trans, diag, A, lda, i, i);       \
            }                                                                       \
            for (long i = 0; i < M; ++i) B[at(order, i, j, ldb)] = (T)x[i];         \
            free(x);                                                                \
        }                                                                           \
    } else {                                                                        \
        _Pragma("omp parallel for schedule(dynamic, 1)")                            \
        for (long i = 0; i < M; ++i) {                                              \
            double *x = (double *)malloc((size_t)N * sizeof(double));               \
            for (long t = 0; t < N; ++t) {                                          \
                long c = eff_lower ? N - 1 - t : t;                                 \
                double s = (alpha != 0.0) ? alpha * (double)B[at(order, i, c, ldb)] : 0.0; \
                long l0 = eff_lower ? c + 1 : 0, l1 = eff_lower ? N : c;            \
                for (long l = l0; l < l1; ++l)                                      \
                    s -= x[l] * top_##SFX(order, uplo, trans, diag, A, lda, l, c);  \
                x[c] = s / top_##SFX(order, uplo, trans, diag, A, lda, c, c);       \
            }                                                                       \
            for (long c = 0; c < N; ++c) B[at(order, i, c, ldb)] = (T)x[c];         \
            free(x);                                                                \
        }                                                                           \
    }                                                                               \
    return 0;                                                                       \
}

DEFINE_TRSM(ref_dtrsm, double, d)
DEFINE_TRSM(ref_strsm, float, s)

int ref_max_threads(void);
#ifdef _OPENMP
#include <omp.h>
int ref_max_threads(void) { return omp_get_max_threads(); }
#else
int ref_max_threads(void) { return 1; }
#endif
