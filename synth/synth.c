/*
 * Seeded synthetic inputs for the tile-BLAS tests and benchmark.
 *
 * This module only fills buffers with pseudo-random numbers.  It holds none of
 * the arithmetic of the method under test; both the CPU oracle side and the
 * GPU side of a test read the very same buffers that these routines fill.
 *
 * The paper's workloads (Section V.A) are dense square matrices with random
 * contents and random scalars; nothing about the values matters beyond being
 * dense and of order one, so an element-addressable uniform[-1,1) generator
 * stands in for them.
 *
 * Generator: element (i, j) of matrix number `mat` (0 = A, 1 = B, 2 = C, ...)
 * with `rows` logical rows under seed s is
 *     u   = mix64(s * 0x9E3779B97F4A7C15 + (mat << 60) + i + j * rows)
 *     val = 2 * (u >> 11) * 2^-53 - 1            in [-1, 1)
 * where mix64 is the splitmix64 output function.  Any element can be
 * regenerated without materialising the matrix.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline double unit_pm1(uint64_t seed, uint64_t mat, uint64_t i, uint64_t j, uint64_t rows)
{
    uint64_t u = mix64(seed * 0x9E3779B97F4A7C15ull + (mat << 60) + i + j * rows);
    return 2.0 * ((double)(u >> 11) * 0x1.0p-53) - 1.0;
}

/* One element, for spot checks from Python. */
double synth_element(uint64_t seed, int mat, int64_t i, int64_t j, int64_t rows)
{
    return unit_pm1(seed, (uint64_t)mat, (uint64_t)i, (uint64_t)j, (uint64_t)rows);
}

/* Column-major rows x cols block with leading dimension ld (elements). */
void synth_fill_f64(double *p, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cols; ++j) {
        double *col = p + (size_t)j * (size_t)ld;
        for (int64_t i = 0; i < rows; ++i)
            col[i] = unit_pm1(seed, (uint64_t)mat, (uint64_t)i, (uint64_t)j, (uint64_t)rows);
    }
}

void synth_fill_f32(float *p, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cols; ++j) {
        float *col = p + (size_t)j * (size_t)ld;
        for (int64_t i = 0; i < rows; ++i)
            col[i] = (float)unit_pm1(seed, (uint64_t)mat, (uint64_t)i, (uint64_t)j, (uint64_t)rows);
    }
}

/* The nr x nc block at (r0, c0) of the rows x (anything) matrix that synth_fill_* would make,
 * regenerated on its own into a column-major buffer with leading dimension ld. */
void synth_block_f64(double *p, int64_t r0, int64_t c0, int64_t nr, int64_t nc, int64_t ld, int64_t rows, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < nc; ++j)
        for (int64_t i = 0; i < nr; ++i)
            p[(size_t)i + (size_t)j * (size_t)ld] = unit_pm1(seed, (uint64_t)mat, (uint64_t)(r0 + i), (uint64_t)(c0 + j), (uint64_t)rows);
}

void synth_block_f32(float *p, int64_t r0, int64_t c0, int64_t nr, int64_t nc, int64_t ld, int64_t rows, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < nc; ++j)
        for (int64_t i = 0; i < nr; ++i)
            p[(size_t)i + (size_t)j * (size_t)ld] = (float)unit_pm1(seed, (uint64_t)mat, (uint64_t)(r0 + i), (uint64_t)(c0 + j), (uint64_t)rows);
}

/*
 * Overwrite the diagonal of an n x n column-major matrix with n + uniform[0,1)
 * so that a triangle of it is strongly diagonally dominant (the triangular
 * workloads: well conditioned, no growth in substitution).
 */
void synth_dominant_diag_f64(double *p, int64_t n, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double u = 0.5 * (unit_pm1(seed ^ 0xD1A6ull, (uint64_t)mat, (uint64_t)i, (uint64_t)i, (uint64_t)n) + 1.0);
        p[(size_t)i + (size_t)i * (size_t)ld] = (double)n + u;
    }
}

void synth_dominant_diag_f32(float *p, int64_t n, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double u = 0.5 * (unit_pm1(seed ^ 0xD1A6ull, (uint64_t)mat, (uint64_t)i, (uint64_t)i, (uint64_t)n) + 1.0);
        p[(size_t)i + (size_t)i * (size_t)ld] = (float)((double)n + u);
    }
}

/* Small integers in {-2,...,2}: products and sums stay exact in floating point. */
void synth_fill_int_f64(double *p, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cols; ++j) {
        double *col = p + (size_t)j * (size_t)ld;
        for (int64_t i = 0; i < rows; ++i) {
            uint64_t u = mix64(seed * 0x9E3779B97F4A7C15ull + ((uint64_t)mat << 60) + (uint64_t)i + (uint64_t)j * (uint64_t)rows);
            col[i] = (double)((int64_t)(u % 5ull) - 2);
        }
    }
}

void synth_fill_int_f32(float *p, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, int mat)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cols; ++j) {
        float *col = p + (size_t)j * (size_t)ld;
        for (int64_t i = 0; i < rows; ++i) {
            uint64_t u = mix64(seed * 0x9E3779B97F4A7C15ull + ((uint64_t)mat << 60) + (uint64_t)i + (uint64_t)j * (uint64_t)rows);
            col[i] = (float)((int64_t)(u % 5ull) - 2);
        }
    }
}
