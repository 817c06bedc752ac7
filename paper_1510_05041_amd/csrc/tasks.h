// Task-ization of the level-3 routines (paper Section IV.A): the output matrix is virtually
// cut into T x T tiles (Section III.A; edge tiles are smaller), and solving one output tile
// C_ij is one task.  A task only holds metadata: tile indices, tile extents, host addresses
// and the list of (A_ik, B_kj) operand tiles its k-steps need (Eq. 1a-1d).  A transposed
// operand is expressed by fetching the mirrored stored tile and flagging the kernel to
// transpose it on the fly (Section III.C).
//
// Everything here is column-major; the C entry points rewrite row-major calls first.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "tile_step.h"

namespace blasx {

// A tile as it is stored in a host matrix.
struct TileRef {
    const char* host = nullptr;  // address of its first element
    int64_t ld = 0;              // host leading dimension (elements)
    int32_t rows = 0, cols = 0;  // stored extent
};

struct StepSpec {
    TileRef a, b;        // left and right operand tiles (as stored)
    int32_t k = 0;       // inner extent of this step
    uint32_t seg_flags = 0;  // TS_TRI_* when one operand is a diagonal tile of a triangular matrix
    int32_t dep = -1;    // index of the task whose *result* one operand is (TRSM), or -1
    bool a_is_dep = false, b_is_dep = false;
    // SYMM: the operand is a diagonal tile of a symmetric matrix of which only one triangle is
    // stored; the kernel gets a device copy with the other triangle filled in by reflection.
    bool a_sym = false, b_sym = false;
    bool sym_lower = false;
    // SYMM: the operand is the transpose of the stored tile (a tile of the symmetric matrix that
    // lies outside the stored triangle); the kernel gets a transposed device copy.
    bool a_mirror = false, b_mirror = false;
};

struct Task {
    int32_t ti = 0, tj = 0;      // tile indices of the output tile
    int32_t m = 0, n = 0;        // its extent
    char* c_host = nullptr;      // host address of the output tile
    bool load_c = false;         // fetch the host tile before the first step
    double alpha_step = 1.0;     // multiplies every step's product
    double beta_first = 0.0;     // multiplies the fetched tile on the first step (later steps: 1)
    uint32_t c_flags = 0;        // TS_C_LOWER / TS_C_UPPER for diagonal tiles of SYRK
    std::vector<StepSpec> steps;
    // TRSM: after the steps, the tile is multiplied by the inverse of this diagonal tile.
    bool solve = false;
    bool solve_on_right = false; // X * inv(op(A_jj)) instead of inv(op(A_ii)) * X
    TileRef diag;
    uint32_t diag_flags = 0;     // TS_TRI_LOWER / TS_TRI_UNIT of the stored diagonal tile
    int32_t panel = -1;          // TRMM: index into Problem::panels (snapshot group), else -1
    double flops = 0.0;
};

// TRMM overwrites the matrix its tasks read.  All tasks of one panel (a tile column for
// Side = left, a tile row for right) read only tiles of that panel, so the panel's original
// tiles are fetched and pinned before its first task starts, and its write-backs are ordered
// after those fetches.
struct Panel {
    std::vector<TileRef> tiles;
    int32_t ntasks = 0;
};

struct Problem {
    int dtype = 0;           // 0 = fp64, 1 = fp32
    size_t esize = 8;
    bool ta = false, tb = false;   // kernel transposes its left / right operand
    int64_t ldc = 0;         // host leading dimension of the output matrix
    const void* c_host = nullptr;      // the output matrix as stored (column-major): first element,
    int64_t c_rows = 0, c_cols = 0;    // and extent
    int T = 0;
    bool results_are_operands = false;  // TRSM: finished tiles stay cached under their host address
    int steps_per_k = 1;     // k-steps a task makes per tile of the inner dimension (SYR2K: 2)
    std::vector<Task> tasks; // in queue order
    std::vector<Panel> panels;
    double flops = 0.0;
};

struct OrderOpts {
    int sb_rows = 4, sb_cols = 4;   // super-block shape for the queue order
    int shells = 1;                 // 1: super-blocks in growing square shells, 0: row by row (serpentine)
};

// C (M x N) <- alpha op(A) op(B) + beta C.
void build_gemm(Problem& p, int dtype, int T, bool ta, bool tb, int M, int N, int K, double alpha,
                const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                const OrderOpts& oo);
// Triangle `lower` of C (N x N) <- alpha A A^T + beta C (trans = false, A N x K) or alpha A^T A + beta C.
void build_syrk(Problem& p, int dtype, int T, bool lower, bool trans, int N, int K, double alpha,
                const void* A, int64_t lda, double beta, void* C, int64_t ldc, const OrderOpts& oo);
// Triangle `lower` of C (N x N) <- alpha (A B^T + B A^T) + beta C (trans = false) or alpha (A^T B + B^T A) + beta C.
void build_syr2k(Problem& p, int dtype, int T, bool lower, bool trans, int N, int K, double alpha,
                 const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                 const OrderOpts& oo);
// C (M x N) <- alpha A B + beta C (left, A M x M symmetric) or alpha B A + beta C (right, A N x N symmetric);
// only the `lower` (or upper) triangle of A is stored.
void build_symm(Problem& p, int dtype, int T, bool left, bool lower, int M, int N, double alpha,
                const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                const OrderOpts& oo);
// B (M x N) <- alpha op(A) B (left) or alpha B op(A) (right).
void build_trmm(Problem& p, int dtype, int T, bool left, bool lower, bool trans, bool unit, int M, int N,
                double alpha, const void* A, int64_t lda, void* B, int64_t ldb, const OrderOpts& oo);
// Solve op(A) X = alpha B (left) or X op(A) = alpha B (right); X overwrites B.
void build_trsm(Problem& p, int dtype, int T, bool left, bool lower, bool trans, bool unit, int M, int N,
                double alpha, const void* A, int64_t lda, void* B, int64_t ldb, const OrderOpts& oo);

// Section III.A: how many square and non-square tiles a rows x cols matrix has.
void tile_counts(int64_t rows, int64_t cols, int T, int64_t* square, int64_t* nonsquare);

}  // namespace blasx
