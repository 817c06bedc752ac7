// C ABI of the tile level-3 BLAS: argument checking, BLAS quick returns, row-major to
// column-major rewriting, then task-ization and the scheduler run.  See include/blasx.h.
#include "../../include/blasx.h"

#include <algorithm>
#include <cstring>
#include <memory>
#include <string>

#include "backend.h"
#include "scheduler.h"
#include "tasks.h"

using namespace blasx;

namespace {

struct Library {
    std::unique_ptr<Backend> be;
    // the same streams over the statically allocated tile arena, with a fixed pool of events: what the
    // allocation-free entry point runs on
    std::unique_ptr<Backend> be_static;
    int T = 1024;
    size_t cache_cap = 0;
    SchedConfig cfg;
    OrderOpts order;
    Stats stats;
    std::string last_error;
    // "persist" = 1: one scheduler, and with it the tile cache, lives across calls
    bool persist = false;
    std::unique_ptr<Scheduler> sched;
    size_t sched_slot_bytes = 0, sched_nslots = 0;
    int sched_T = 0;
    int last_T = 0;   // tile edge of the most recent call
    int last_group = 0;
    bool last_wide = false;
    int last_ramp = 0;
    int last_kchain = 0;
};

Library& lib() {
    static Library L;
    return L;
}

// Tile edge for one call: the configured one, or (tile = 0) chosen from the extent of the output matrix,
// the element type and the room in the tile cache.  The rules (measured end to end on an MI355X with
// paper_1510_05041_amd/tune.py; the tables are in profiles/tile_stream_sweep_mi355x.md):
//   - a tile must be large enough that the fixed cost of one strided copy (~10 us on the copy engine) is
//     small beside its transfer time: 1024 (8 MB) in double precision from 2048 rows or columns up, one tile
//     per matrix below; larger tiles only shorten the k loop that the wide schedule pipelines;
//   - single precision: 2048 (the same 16 MB) from 6656 up, but 1024 where the wide schedule applies or nearly
//     (output and inner dimension from 11264), below 6656, and for the triangular product throughout; 2048 again
//     where every tile of C is a task (GEMM, SYMM) and all three extents reach 28672: such a call is bound by
//     the kernel, and launches of four times the work each have less fixed cost to pay;
//   - `solve_order` (order of the triangular matrix of a TRSM, else 0): the wide solve advances one k-tile per
//     round, so its update launches are one tile deep, and from 20 tiles of 1024 on the twice as deep launches
//     of 2048-tiles win (double precision from 20480; single precision above 12288, 1024 from 4097);
//   - small triangular calls take the tile that gives them the five block rows from which the wide schedule
//     runs: 512 for orders 2560 .. 4096 (TRSM in both precisions, DTRMM);
//   - halved until 64 tiles fit the cache (running set + operands), else eviction thrashes.
int pick_tile(int dtype, int64_t rows, int64_t cols, int64_t inner, int64_t solve_order = 0, bool tri_product = false,
              bool full_output = false) {
    Library& L = lib();
    if (L.T > 0) return L.T;
    const int64_t n = std::max<int64_t>(1, std::max(rows, cols));
    const size_t es = dtype == 0 ? 8 : 4;
    const int64_t one_tile = (n + 15) / 16 * 16;
    const bool five_rows_of_512 = solve_order >= 2560 && solve_order <= 4096;
    int T;
    if (dtype == 0) {
        if (solve_order >= 20480) T = 2048;
        else if (five_rows_of_512 || (tri_product && inner >= 2560 && inner <= 4096)) T = 512;
        else T = n >= 2048 ? 1024 : (int)one_tile;
    } else {
        if (solve_order > 12288) T = 2048;
        else if (five_rows_of_512) T = 512;
        else if (solve_order > 4096) T = 1024;
        else if (full_output && std::min(rows, cols) >= 28672 && inner >= 28672) T = 2048;
        else if (n >= 11264 && inner >= 11264) T = 1024;
        else if (n >= 6656 && !tri_product) T = 2048;
        else T = n > 2048 ? 1024 : (int)std::min<int64_t>(2048, one_tile);
    }
    // at least 64 tiles must fit in the cache (running set + operands), else eviction thrashes
    size_t usable = L.be ? L.be->arena_bytes() : 0;
    if (L.cache_cap && L.cache_cap < usable) usable = L.cache_cap;
    while (usable && T > 256 && usable / ((size_t)T * T * es) < 64) T = std::max(256, (T / 2 + 15) / 16 * 16);
    return T;
}

// Number of tile tasks that run together.  Many tasks in lockstep fill the chip with one launch but also
// finish together: their write-backs bunch up at the end and the first launch waits for the first tiles of
// all of them.  When the call is bound by the link (few tiles per dimension) a small running set pipelines
// better.  Rule (tables in profiles/tile_stream_sweep_mi355x.md): one twelfth of the task count as a power
// of two in 2..16, for the rectangular and the triangular task sets alike.
int pick_group(const Problem& p) {
    Library& L = lib();
    if (L.cfg.group > 0) return L.cfg.group;
    if (!p.panels.empty() || p.results_are_operands) return 16;   // TRMM / TRSM: parallelism is per dependency level
    size_t want = std::min<size_t>(16, std::max<size_t>(2, p.tasks.size() / 12));
    // from 5 x 5 tiles of up to 8 MB at least 4 (not for tiles of 16 MB, whose copies take twice as long)
    const int64_t side = std::max((p.c_rows + p.T - 1) / p.T, (p.c_cols + p.T - 1) / p.T);
    const bool big_tiles = (size_t)p.T * p.T * p.esize > ((size_t)8 << 20);
    if (side >= 5 && !big_tiles) want = std::max<size_t>(want, 4);
    // a k loop too short for the wide schedule (many output tiles, few k-tiles): the call is bound by the link, and
    // 8 tasks pipeline better than 16 (tiles of 16 MB: 4)
    size_t longest = 0;
    for (const Task& t : p.tasks) longest = std::max(longest, t.steps.size());
    if (L.cfg.wide > 0 && longest < (size_t)L.cfg.wide * (size_t)p.steps_per_k) want = std::min<size_t>(want, big_tiles ? 4 : 8);
    int g = 2;
    while ((size_t)g * 2 <= want) g *= 2;
    return g;
}

bool is_trans(int t) { return t == BLASX_TRANS || t == BLASX_CONJ_TRANS; }
bool ok_trans(int t) { return t == BLASX_NO_TRANS || is_trans(t); }

constexpr int kStaticTile = 512;        // largest tile edge of the allocation-free entry point
constexpr int kStaticEvents = 1024;     // its event pool: a fill event per slot, one per launch in flight and per pending result

size_t slot_bytes_of(int T, size_t esize) { return ((size_t)T * (size_t)T * esize + 255) / 256 * 256; }

// on_static: run on the statically allocated arena (whole of it, no cap, cache dropped at return)
int run_problem(Problem& p, bool on_static = false) {
    Library& L = lib();
    Backend& be = on_static ? *L.be_static : *L.be;
    L.last_T = p.T;
    const size_t slot_bytes = slot_bytes_of(p.T, p.esize);
    size_t usable = be.arena_bytes();
    if (!on_static && L.cache_cap && L.cache_cap < usable) usable = L.cache_cap;
    const size_t nslots = usable / slot_bytes;
    if (nslots < 4) {
        L.last_error = "tile cache holds fewer than 4 tiles of the configured size";
        return BLASX_ERR_ARENA_TOO_SMALL;
    }
    SchedConfig cfg = L.cfg;
    if (on_static) cfg.profile = 0;      // event-timed launches would draw on the fixed event pool
    cfg.group = pick_group(p);
    cfg.rs = std::max(cfg.rs, 2 * cfg.group);
    // the running set and its operands must fit: each running task owns an accumulator slot
    cfg.group = (int)std::max<size_t>(1, std::min<size_t>((size_t)cfg.group, nslots / 4));
    // TRMM pins the original tiles of the panel of every running task: in the worst case each running task
    // belongs to a panel of its own, and they must all fit beside the tasks' own slots and operands
    size_t panel_tiles = 0;
    for (const Panel& pn : p.panels) panel_tiles = std::max(panel_tiles, pn.tiles.size());
    if (panel_tiles) cfg.group = (int)std::max<size_t>(1, std::min<size_t>((size_t)cfg.group, nslots / (panel_tiles + 4)));
    L.last_group = cfg.group;
    ++L.stats.calls;
    int rc;
    const size_t ns = std::min<size_t>(nslots, 1u << 30);
    if (on_static) {
        Scheduler sched(be, (int)ns, slot_bytes, cfg, L.stats);
        rc = sched.run(p);
        L.last_wide = sched.last_run_was_wide();
        L.last_kchain = sched.last_run_kchain();
        L.last_ramp = sched.last_run_first_chain();
    } else if (L.persist) {
        // the cached tiles survive as long as the slot geometry does
        if (!L.sched || L.sched_slot_bytes != slot_bytes || L.sched_nslots != ns || L.sched_T != p.T) {
            L.sched.reset(new Scheduler(*L.be, (int)ns, slot_bytes, cfg, L.stats));
            L.sched_slot_bytes = slot_bytes;
            L.sched_nslots = ns;
            L.sched_T = p.T;
        }
        L.sched->set_config(cfg);
        rc = L.sched->run(p);
        L.last_wide = L.sched->last_run_was_wide();
        L.last_kchain = L.sched->last_run_kchain();
        L.last_ramp = L.sched->last_run_first_chain();
        if (rc != 0) L.sched.reset();      // after a failed call nothing cached is trusted: start afresh
    } else {
        L.sched.reset();
        Scheduler sched(*L.be, (int)ns, slot_bytes, cfg, L.stats);
        rc = sched.run(p);
        L.last_wide = sched.last_run_was_wide();
        L.last_kchain = sched.last_run_kchain();
        L.last_ramp = sched.last_run_first_chain();
    }
    if (rc == BLASX_ERR_DEVICE) L.last_error = be.last_error();
    if (rc == BLASX_ERR_ARENA_TOO_SMALL) L.last_error = "tile cache too small for the working set of this call";
    return rc;
}

template <typename T>
int gemm_impl(int dtype, int Order, int TransA, int TransB, int M, int N, int K, double alpha, const T* A, int lda,
              const T* B, int ldb, double beta, T* C, int ldc, bool no_alloc = false) {
    if (Order != BLASX_ROW_MAJOR && Order != BLASX_COL_MAJOR) return -1;
    if (!ok_trans(TransA)) return -2;
    if (!ok_trans(TransB)) return -3;
    if (M < 0) return -4;
    if (N < 0) return -5;
    if (K < 0) return -6;
    // stored extents in the order's own terms: rows of A as stored (column-major) / columns (row-major)
    const bool col = Order == BLASX_COL_MAJOR;
    const int a_lead = col ? (is_trans(TransA) ? K : M) : (is_trans(TransA) ? M : K);
    const int b_lead = col ? (is_trans(TransB) ? N : K) : (is_trans(TransB) ? K : N);
    const int c_lead = col ? M : N;
    if (lda < std::max(1, a_lead)) return -9;
    if (ldb < std::max(1, b_lead)) return -11;
    if (ldc < std::max(1, c_lead)) return -14;
    if (M == 0 || N == 0) return 0;
    if ((alpha == 0.0 || K == 0) && beta == 1.0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    if ((!A || !B) && alpha != 0.0 && K > 0) return A ? -10 : -8;
    if (!C) return -13;
    int T_call = 0;
    if (no_alloc) {
        Library& L = lib();
        if (!L.be_static) {
            L.last_error = "the statically allocated tile arena could not be set up by blasx_init";
            return BLASX_ERR_DEVICE;
        }
        const bool reads_ab = alpha != 0.0 && K > 0;
        if ((reads_ab && (!backend_host_is_pinned(A) || !backend_host_is_pinned(B))) || !backend_host_is_pinned(C)) {
            L.last_error = "the allocation-free entry point needs page-locked matrices (the runtime stages pageable memory through buffers of its own)";
            return BLASX_ERR_UNSUPPORTED;
        }
        // every tile of A, B and C must have a slot of its own (plus the few the pipeline holds besides): nothing is
        // ever evicted, and the call is refused rather than squeezed
        T_call = L.T > 0 && L.T < kStaticTile ? L.T : kStaticTile;
        auto nt = [&](int64_t x) { return (size_t)((x + T_call - 1) / T_call); };
        const size_t tiles = (reads_ab ? nt(M) * nt(K) + nt(K) * nt(N) : 0) + nt(M) * nt(N);
        const size_t slots = L.be_static->arena_bytes() / slot_bytes_of(T_call, sizeof(T));
        if (tiles + 8 > slots) {
            L.last_error = "too large for the allocation-free entry point: " + std::to_string(tiles) + " tiles of " + std::to_string(T_call) +
                           " x " + std::to_string(T_call) + " (+ 8) against " + std::to_string(slots) + " slots of static scratch";
            return BLASX_ERR_TOO_LARGE;
        }
    } else {
        T_call = pick_tile(dtype, M, N, K, 0, false, true);
    }
    Problem p;
    if (col)
        build_gemm(p, dtype, T_call, is_trans(TransA), is_trans(TransB), M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, lib().order);
    else   // C^T = op(B)^T op(A)^T: the row-major arrays are the column-major transposes
        build_gemm(p, dtype, T_call, is_trans(TransB), is_trans(TransA), N, M, K, alpha, B, ldb, A, lda, beta, C, ldc, lib().order);
    return run_problem(p, no_alloc);
}

int tri_check(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, const void* A, int lda, const void* B,
              int ldb) {
    if (Order != BLASX_ROW_MAJOR && Order != BLASX_COL_MAJOR) return -1;
    if (Side != BLASX_LEFT && Side != BLASX_RIGHT) return -2;
    if (Uplo != BLASX_UPPER && Uplo != BLASX_LOWER) return -3;
    if (!ok_trans(TransA)) return -4;
    if (Diag != BLASX_NON_UNIT && Diag != BLASX_UNIT) return -5;
    if (M < 0) return -6;
    if (N < 0) return -7;
    const int na = Side == BLASX_LEFT ? M : N;
    if (lda < std::max(1, na)) return -10;
    if (ldb < std::max(1, Order == BLASX_COL_MAJOR ? M : N)) return -12;
    if (M > 0 && N > 0) {
        if (!A) return -9;
        if (!B) return -11;
    }
    return 0;
}

int syrk_impl(int dtype, int Order, int Uplo, int Trans, int N, int K, double alpha, const void* A, int lda, double beta,
              void* C, int ldc) {
    if (Order != BLASX_ROW_MAJOR && Order != BLASX_COL_MAJOR) return -1;
    if (Uplo != BLASX_UPPER && Uplo != BLASX_LOWER) return -2;
    if (!ok_trans(Trans)) return -3;
    if (N < 0) return -4;
    if (K < 0) return -5;
    const bool col = Order == BLASX_COL_MAJOR;
    const int a_lead = col ? (is_trans(Trans) ? K : N) : (is_trans(Trans) ? N : K);
    if (lda < std::max(1, a_lead)) return -8;
    if (ldc < std::max(1, N)) return -11;
    if (N == 0) return 0;
    if ((alpha == 0.0 || K == 0) && beta == 1.0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    if (!A && alpha != 0.0 && K > 0) return -7;
    if (!C) return -10;
    Problem p;
    // row-major: the arrays are the column-major transposes, so the triangle and the
    // transposition flag both flip
    const bool lower = col ? (Uplo == BLASX_LOWER) : (Uplo == BLASX_UPPER);
    const bool trans = col ? is_trans(Trans) : !is_trans(Trans);
    build_syrk(p, dtype, pick_tile(dtype, N, N, K), lower, trans, N, K, alpha, A, lda, beta, C, ldc, lib().order);
    return run_problem(p);
}

int syr2k_impl(int dtype, int Order, int Uplo, int Trans, int N, int K, double alpha, const void* A, int lda, const void* B,
               int ldb, double beta, void* C, int ldc) {
    if (Order != BLASX_ROW_MAJOR && Order != BLASX_COL_MAJOR) return -1;
    if (Uplo != BLASX_UPPER && Uplo != BLASX_LOWER) return -2;
    if (!ok_trans(Trans)) return -3;
    if (N < 0) return -4;
    if (K < 0) return -5;
    const bool col = Order == BLASX_COL_MAJOR;
    const int ab_lead = col ? (is_trans(Trans) ? K : N) : (is_trans(Trans) ? N : K);
    if (lda < std::max(1, ab_lead)) return -8;
    if (ldb < std::max(1, ab_lead)) return -10;
    if (ldc < std::max(1, N)) return -13;
    if (N == 0) return 0;
    if ((alpha == 0.0 || K == 0) && beta == 1.0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    if ((!A || !B) && alpha != 0.0 && K > 0) return A ? -9 : -7;
    if (!C) return -12;
    Problem p;
    const bool lower = col ? (Uplo == BLASX_LOWER) : (Uplo == BLASX_UPPER);
    const bool trans = col ? is_trans(Trans) : !is_trans(Trans);
    build_syr2k(p, dtype, pick_tile(dtype, N, N, K), lower, trans, N, K, alpha, A, lda, B, ldb, beta, C, ldc, lib().order);
    return run_problem(p);
}

int symm_impl(int dtype, int Order, int Side, int Uplo, int M, int N, double alpha, const void* A, int lda, const void* B,
              int ldb, double beta, void* C, int ldc) {
    if (Order != BLASX_ROW_MAJOR && Order != BLASX_COL_MAJOR) return -1;
    if (Side != BLASX_LEFT && Side != BLASX_RIGHT) return -2;
    if (Uplo != BLASX_UPPER && Uplo != BLASX_LOWER) return -3;
    if (M < 0) return -4;
    if (N < 0) return -5;
    const bool col = Order == BLASX_COL_MAJOR;
    const int na = Side == BLASX_LEFT ? M : N;
    const int bc_lead = col ? M : N;
    if (lda < std::max(1, na)) return -8;
    if (ldb < std::max(1, bc_lead)) return -10;
    if (ldc < std::max(1, bc_lead)) return -13;
    if (M == 0 || N == 0) return 0;
    if (alpha == 0.0 && beta == 1.0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    if ((!A || !B) && alpha != 0.0) return A ? -9 : -7;
    if (!C) return -12;
    Problem p;
    // row-major: C^T = alpha (A B)^T = alpha B^T A: side and triangle flip, M and N swap
    const bool left = col ? (Side == BLASX_LEFT) : (Side == BLASX_RIGHT);
    const bool lower = col ? (Uplo == BLASX_LOWER) : (Uplo == BLASX_UPPER);
    build_symm(p, dtype, pick_tile(dtype, M, N, Side == BLASX_LEFT ? M : N, 0, false, true), left, lower, col ? M : N, col ? N : M, alpha, A, lda, B, ldb, beta, C, ldc, lib().order);
    return run_problem(p);
}

int trmm_impl(int dtype, int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha, const void* A,
              int lda, void* B, int ldb) {
    const int chk = tri_check(Order, Side, Uplo, TransA, Diag, M, N, A, lda, B, ldb);
    if (chk) return chk;
    if (M == 0 || N == 0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    const bool col = Order == BLASX_COL_MAJOR;
    // row-major: B^T = alpha (op(A) B)^T = alpha B^T op(A)^T: side and triangle flip, M and N swap
    const bool left = col ? (Side == BLASX_LEFT) : (Side == BLASX_RIGHT);
    const bool lower = col ? (Uplo == BLASX_LOWER) : (Uplo == BLASX_UPPER);
    Problem p;
    // the k loop of the triangular product is as long as the triangular matrix is wide
    build_trmm(p, dtype, pick_tile(dtype, M, N, Side == BLASX_LEFT ? M : N, 0, true), left, lower, is_trans(TransA), Diag == BLASX_UNIT, col ? M : N, col ? N : M, alpha, A, lda, B,
               ldb, lib().order);
    return run_problem(p);
}

int trsm_impl(int dtype, int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha, const void* A,
              int lda, void* B, int ldb) {
    const int chk = tri_check(Order, Side, Uplo, TransA, Diag, M, N, A, lda, B, ldb);
    if (chk) return chk;
    if (M == 0 || N == 0) return 0;
    if (!lib().be) return BLASX_ERR_NOT_INITIALIZED;
    const bool col = Order == BLASX_COL_MAJOR;
    const bool left = col ? (Side == BLASX_LEFT) : (Side == BLASX_RIGHT);
    const bool lower = col ? (Uplo == BLASX_LOWER) : (Uplo == BLASX_UPPER);
    Problem p;
    if (alpha == 0.0) {
        // X = 0 and A is not read: a TRMM with no steps writes zero tiles
        build_trmm(p, dtype, pick_tile(dtype, M, N, 0), left, lower, is_trans(TransA), Diag == BLASX_UNIT, col ? M : N, col ? N : M, 0.0, A, lda, B,
                   ldb, lib().order);
    } else {
        build_trsm(p, dtype, pick_tile(dtype, M, N, 0, Side == BLASX_LEFT ? M : N), left, lower, is_trans(TransA), Diag == BLASX_UNIT, col ? M : N, col ? N : M, alpha, A, lda, B,
                   ldb, lib().order);
    }
    return run_problem(p);
}

}  // namespace

extern "C" {

int blasx_dgemm(int Order, int TransA, int TransB, int M, int N, int K, double alpha, const double* A, int lda,
                const double* B, int ldb, double beta, double* C, int ldc) {
    return gemm_impl<double>(0, Order, TransA, TransB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
}

int blasx_dgemm_noalloc(int Order, int TransA, int TransB, int M, int N, int K, double alpha, const double* A, int lda,
                        const double* B, int ldb, double beta, double* C, int ldc) {
    return gemm_impl<double>(0, Order, TransA, TransB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, true);
}

int blasx_sgemm(int Order, int TransA, int TransB, int M, int N, int K, float alpha, const float* A, int lda,
                const float* B, int ldb, float beta, float* C, int ldc) {
    return gemm_impl<float>(1, Order, TransA, TransB, M, N, K, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc);
}

int blasx_dsyrk(int Order, int Uplo, int Trans, int N, int K, double alpha, const double* A, int lda, double beta,
                double* C, int ldc) {
    return syrk_impl(0, Order, Uplo, Trans, N, K, alpha, A, lda, beta, C, ldc);
}
int blasx_ssyrk(int Order, int Uplo, int Trans, int N, int K, float alpha, const float* A, int lda, float beta,
                float* C, int ldc) {
    return syrk_impl(1, Order, Uplo, Trans, N, K, (double)alpha, A, lda, (double)beta, C, ldc);
}

int blasx_dsyr2k(int Order, int Uplo, int Trans, int N, int K, double alpha, const double* A, int lda, const double* B,
                 int ldb, double beta, double* C, int ldc) {
    return syr2k_impl(0, Order, Uplo, Trans, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
}
int blasx_ssyr2k(int Order, int Uplo, int Trans, int N, int K, float alpha, const float* A, int lda, const float* B, int ldb,
                 float beta, float* C, int ldc) {
    return syr2k_impl(1, Order, Uplo, Trans, N, K, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc);
}

int blasx_dsymm(int Order, int Side, int Uplo, int M, int N, double alpha, const double* A, int lda, const double* B, int ldb,
                double beta, double* C, int ldc) {
    return symm_impl(0, Order, Side, Uplo, M, N, alpha, A, lda, B, ldb, beta, C, ldc);
}
int blasx_ssymm(int Order, int Side, int Uplo, int M, int N, float alpha, const float* A, int lda, const float* B, int ldb,
                float beta, float* C, int ldc) {
    return symm_impl(1, Order, Side, Uplo, M, N, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc);
}

int blasx_dtrmm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha, const double* A, int lda,
                double* B, int ldb) {
    return trmm_impl(0, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb);
}
int blasx_strmm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, float alpha, const float* A, int lda,
                float* B, int ldb) {
    return trmm_impl(1, Order, Side, Uplo, TransA, Diag, M, N, (double)alpha, A, lda, B, ldb);
}

int blasx_dtrsm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha, const double* A, int lda,
                double* B, int ldb) {
    return trsm_impl(0, Order, Side, Uplo, TransA, Diag, M, N, alpha, A, lda, B, ldb);
}
int blasx_strsm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, float alpha, const float* A, int lda,
                float* B, int ldb) {
    return trsm_impl(1, Order, Side, Uplo, TransA, Diag, M, N, (double)alpha, A, lda, B, ldb);
}

int blasx_init(void* arena, size_t arena_bytes, void* const* hip_streams, int nstreams) {
    Library& L = lib();
    L.sched.reset();
    L.be_static.reset();
    L.be.reset();
    if (nstreams == 0) nstreams = 4;   // measured best at every size (a second inbound stream hides per-copy latency)
    if (nstreams < 2 || nstreams > 4 || arena_bytes == 0) return BLASX_ERR_CONFIG;
    std::string err;
    Backend* b = make_backend(arena, arena_bytes, hip_streams, nstreams, &err);
    if (!b) {
        L.last_error = err;
        return BLASX_ERR_DEVICE;
    }
    L.be.reset(b);
    // Set-up of the allocation-free entry point, here so that the entry point itself creates nothing: the device
    // address of this GPU's statically allocated arena, the same streams over it, a fixed pool of events, and the
    // double-precision kernels loaded.  A failure is not an error of blasx_init; the entry point reports it.
    void* sptr = nullptr;
    size_t sbytes = 0;
    if (backend_static_arena(&sptr, &sbytes) == 0) {
        std::string serr;
        std::unique_ptr<Backend> s(make_backend(sptr, sbytes, hip_streams, nstreams, &serr));
        if (s && s->reserve_events(kStaticEvents) == 0 && backend_warm_kernels(*s, 0) == 0) L.be_static = std::move(s);
    }
    return 0;
}

int blasx_shutdown(void) {
    lib().sched.reset();
    lib().be_static.reset();
    lib().be.reset();
    backend_release_device_memory();
    return 0;
}

int blasx_set_tile(int T) {
    if (T != 0 && (T < 16 || T > 8192 || T % 16)) return BLASX_ERR_CONFIG;
    lib().T = T;
    return 0;
}

int blasx_set_streams(int n) {
    Library& L = lib();
    if (!L.be) return BLASX_ERR_NOT_INITIALIZED;
    if (n == 0) n = 4;
    if (L.be->set_num_streams(n)) {
        L.last_error = L.be->last_error();
        return BLASX_ERR_CONFIG;
    }
    if (L.be_static) L.be_static->set_num_streams(n);
    return 0;
}

int blasx_set_cache_bytes(size_t cap) {
    lib().cache_cap = cap;
    return 0;
}

int blasx_set_option(const char* name, long value) {
    if (!name) return BLASX_ERR_CONFIG;
    Library& L = lib();
    const std::string n(name);
    if (n == "group") { if (value < 0 || value > 4096) return BLASX_ERR_CONFIG; L.cfg.group = (int)value; }
    else if (n == "kchain") { if (value < 0 || value > kMaxChain) return BLASX_ERR_CONFIG; L.cfg.kchain = (int)value; }
    else if (n == "depth") { if (value < 1 || value > 1024) return BLASX_ERR_CONFIG; L.cfg.depth = (int)value; }
    else if (n == "rs") { if (value < 1 || value > 65536) return BLASX_ERR_CONFIG; L.cfg.rs = (int)value; }
    else if (n == "priority") { if (value < 0 || value > 1) return BLASX_ERR_CONFIG; L.cfg.priority = value != 0; }
    else if (n == "sb_rows") { if (value < 1 || value > 4096) return BLASX_ERR_CONFIG; L.order.sb_rows = (int)value; }
    else if (n == "sb_cols") { if (value < 1 || value > 4096) return BLASX_ERR_CONFIG; L.order.sb_cols = (int)value; }
    else if (n == "shells") { if (value < 0 || value > 1) return BLASX_ERR_CONFIG; L.order.shells = (int)value; }
    else if (n == "wide") { if (value < 0 || value > 65536) return BLASX_ERR_CONFIG; L.cfg.wide = (int)value; }
    else if (n == "ramp") { if (value < 0 || value > kMaxChain) return BLASX_ERR_CONFIG; L.cfg.ramp = (int)value; }
    else if (n == "prefetch") { if (value < 0 || value > 4096) return BLASX_ERR_CONFIG; L.cfg.prefetch = (int)value; }
    else if (n == "late_c") { if (value < 0 || value > 1) return BLASX_ERR_CONFIG; L.cfg.late_c = value != 0; }
    else if (n == "row_order") { if (value < 0 || value > 1) return BLASX_ERR_CONFIG; L.cfg.row_order = value != 0; }
    else if (n == "tail_cut") { if (value < 0 || value > 16) return BLASX_ERR_CONFIG; L.cfg.tail_cut = (int)value; }
    else if (n == "stagger_panels") { if (value < 1 || value > 64) return BLASX_ERR_CONFIG; L.cfg.stagger_panels = (int)value; }
    else if (n == "stagger_lag") { if (value < -1 || value > 4096) return BLASX_ERR_CONFIG; L.cfg.stagger_lag = (int)value; }
    else if (n == "merge") { if (value < 0 || value > 8) return BLASX_ERR_CONFIG; L.cfg.merge = (int)value; }
    else if (n == "profile") { if (value < 0 || value > 2) return BLASX_ERR_CONFIG; L.cfg.profile = (int)value; }
    else if (n == "persist") {
        if (value < 0 || value > 1) return BLASX_ERR_CONFIG;
        L.persist = value != 0;
        if (!L.persist) L.sched.reset();
    }
    else return BLASX_ERR_CONFIG;
    return 0;
}

long blasx_get_option(const char* name) {
    if (!name) return -1;
    Library& L = lib();
    const std::string n(name);
    if (n == "group") return L.cfg.group;
    if (n == "kchain") return L.cfg.kchain;
    if (n == "depth") return L.cfg.depth;
    if (n == "rs") return L.cfg.rs;
    if (n == "priority") return L.cfg.priority ? 1 : 0;
    if (n == "sb_rows") return L.order.sb_rows;
    if (n == "sb_cols") return L.order.sb_cols;
    if (n == "shells") return L.order.shells;
    if (n == "wide") return L.cfg.wide;
    if (n == "prefetch") return L.cfg.prefetch;
    if (n == "ramp") return L.cfg.ramp;
    if (n == "merge") return L.cfg.merge;
    if (n == "stagger_panels") return L.cfg.stagger_panels;
    if (n == "stagger_lag") return L.cfg.stagger_lag;
    if (n == "tail_cut") return L.cfg.tail_cut;
    if (n == "row_order") return L.cfg.row_order ? 1 : 0;
    if (n == "late_c") return L.cfg.late_c ? 1 : 0;
    if (n == "profile") return L.cfg.profile;
    if (n == "streams") return L.be ? L.be->num_streams() : 0;
    if (n == "persist") return L.persist ? 1 : 0;
    if (n == "cached_tiles") return L.sched ? (long)L.sched->cached_blocks() : 0;
    if (n == "tile") return L.T;
    if (n == "last_tile") return L.last_T;
    if (n == "last_group") return L.last_group;
    if (n == "last_wide") return L.last_wide ? 1 : 0;
    if (n == "last_ramp") return L.last_ramp;
    if (n == "last_kchain") return L.last_kchain;
    return -1;
}

int blasx_invalidate(const void* ptr, size_t bytes) {
    if (!ptr && bytes) return -1;
    Library& L = lib();
    if (L.sched && bytes) L.sched->invalidate_region(ptr, (int64_t)bytes, (int64_t)bytes, 1, 1);
    return 0;
}

int blasx_invalidate_matrix(const void* A, int ld, int rows, int cols, int elem_size) {
    if (rows < 0) return -3;
    if (cols < 0) return -4;
    if (elem_size != 4 && elem_size != 8) return -5;
    if (ld < std::max(1, rows)) return -2;
    if (!A && rows && cols) return -1;
    Library& L = lib();
    if (L.sched && rows && cols) L.sched->invalidate_region(A, ld, rows, cols, elem_size);
    return 0;
}

int blasx_invalidate_all(void) {
    Library& L = lib();
    if (L.sched) L.sched->invalidate_all();
    return 0;
}

void* blasx_host_alloc(size_t bytes) { return backend_host_alloc(bytes); }
int blasx_host_free(void* p) { return backend_host_free(p) ? BLASX_ERR_DEVICE : 0; }

int blasx_get_stats(blasx_stats* out) {
    if (!out) return BLASX_ERR_CONFIG;
    const Stats& s = lib().stats;
    std::memset(out, 0, sizeof(*out));
    out->calls = s.calls; out->tasks = s.tasks; out->tile_steps = s.tile_steps; out->launches = s.launches;
    out->hits = s.hits; out->misses = s.misses; out->evictions = s.evictions; out->refetches = s.refetches;
    out->copies_h2d = s.copies_h2d; out->copies_d2h = s.copies_d2h; out->bytes_h2d = s.bytes_h2d; out->bytes_d2h = s.bytes_d2h;
    out->slot_waits = s.slot_waits; out->peak_slots = s.peak_slots; out->profiled_launches = s.profiled_launches; out->invalidations = s.invalidations;
    out->flops = s.flops; out->t_total_s = s.t_total_s; out->t_issue_s = s.t_issue_s; out->t_kernel_s = s.t_kernel_s;
    out->t_wait_s = s.t_wait_s; out->t_kernel_busy_s = s.t_kernel_busy_s; out->t_copy_unoverlapped_s = s.t_copy_unoverlapped_s;
    out->t_device_span_s = s.t_device_span_s;
    out->steps_general = s.steps_general;
    out->transfers_h2d = s.transfers_h2d;
    return 0;
}

int blasx_reset_stats(void) {
    lib().stats = Stats();
    return 0;
}

const char* blasx_strerror(int rc) {
    if (rc < 0) return "invalid argument (its 1-based position is the negated code)";
    switch (rc) {
        case BLASX_OK: return "success";
        case BLASX_ERR_NOT_INITIALIZED: return "blasx_init has not been called";
        case BLASX_ERR_ARENA_TOO_SMALL: return "tile cache too small";
        case BLASX_ERR_DEVICE: return "device error";
        case BLASX_ERR_CONFIG: return "invalid configuration value";
        case BLASX_ERR_NO_MEMORY: return "out of host memory";
        case BLASX_ERR_UNSUPPORTED: return "not supported";
        case BLASX_ERR_TOO_LARGE: return "problem too large for the allocation-free entry point";
        default: return "unknown error";
    }
}

const char* blasx_last_error(void) { return lib().last_error.c_str(); }

}  // extern "C"
