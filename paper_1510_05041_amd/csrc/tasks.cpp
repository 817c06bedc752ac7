#include "tasks.h"

#include <algorithm>
#include <functional>
#include <map>
#include <utility>

namespace blasx {

namespace {

inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Stored tile (tr, tc) of a column-major Rows x Cols host matrix.
TileRef stored_tile(const void* base, int64_t ld, size_t esize, int T, int tr, int tc, int64_t Rows, int64_t Cols) {
    TileRef t;
    t.host = static_cast<const char*>(base) + ((size_t)tr * T + (size_t)tc * T * (size_t)ld) * esize;
    t.ld = ld;
    t.rows = (int32_t)std::min<int64_t>(T, Rows - (int64_t)tr * T);
    t.cols = (int32_t)std::min<int64_t>(T, Cols - (int64_t)tc * T);
    return t;
}

// Queue order of output tiles: super-blocks of sb_rows x sb_cols tiles, tiles row by row inside a
// super-block, so that tasks that are neighbours in the queue share A row tiles and B column
// tiles.  The super-blocks themselves are visited either block row by block row in a serpentine,
// or in growing square shells (shell s = down block column s, then back along block row s): a
// shell needs one new block row of A and one new block column of B but holds 2s+1 super-blocks,
// so the inbound traffic is spread over the whole run instead of all of B being needed during
// the first block row.
std::vector<std::pair<int, int>> superblock_order(int nti, int ntj, const OrderOpts& oo,
                                                  const std::function<bool(int, int)>& keep) {
    std::vector<std::pair<int, int>> out;
    const int sr = std::max(1, oo.sb_rows), sc = std::max(1, oo.sb_cols);
    const int nbi = cdiv(nti, sr), nbj = cdiv(ntj, sc);
    std::vector<std::pair<int, int>> blocks;
    if (oo.shells) {
        for (int s = 0; s < std::max(nbi, nbj); ++s) {
            if (s < nbj)
                for (int bi = 0; bi <= std::min(s, nbi - 1); ++bi) blocks.emplace_back(bi, s);
            if (s < nbi)
                for (int bj = std::min(s, nbj) - 1; bj >= 0; --bj) blocks.emplace_back(s, bj);
        }
    } else {
        for (int bi = 0; bi < nbi; ++bi)
            for (int q = 0; q < nbj; ++q) blocks.emplace_back(bi, (bi & 1) ? nbj - 1 - q : q);
    }
    for (auto b : blocks)
        for (int i = b.first * sr; i < std::min(nti, (b.first + 1) * sr); ++i)
            for (int j = b.second * sc; j < std::min(ntj, (b.second + 1) * sc); ++j)
                if (keep(i, j)) out.emplace_back(i, j);
    return out;
}

void init_problem(Problem& p, int dtype, int T, bool ta, bool tb, const void* C, int64_t ldc, int64_t rows, int64_t cols) {
    p = Problem();
    p.c_host = C;
    p.c_rows = rows;
    p.c_cols = cols;
    p.dtype = dtype;
    p.esize = dtype == 0 ? 8 : 4;
    p.ta = ta;
    p.tb = tb;
    p.ldc = ldc;
    p.T = T;
}

}  // namespace

void tile_counts(int64_t rows, int64_t cols, int T, int64_t* square, int64_t* nonsquare) {
    const int64_t fl = (rows / T) * (cols / T);
    const int64_t ce = (int64_t)cdiv(rows, T) * cdiv(cols, T);
    *square = fl;
    *nonsquare = ce - fl;
}

// Eq. 1a: C_ij = alpha * sum_k A_ik B_kj + beta * C_ij.
void build_gemm(Problem& p, int dtype, int T, bool ta, bool tb, int M, int N, int K, double alpha,
                const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                const OrderOpts& oo) {
    init_problem(p, dtype, T, ta, tb, C, ldc, M, N);
    const int ntm = cdiv(M, T), ntn = cdiv(N, T), ntk = (alpha == 0.0) ? 0 : cdiv(K, T);
    const int64_t a_rows = ta ? K : M, a_cols = ta ? M : K;   // stored shapes
    const int64_t b_rows = tb ? N : K, b_cols = tb ? K : N;
    for (auto ij : superblock_order(ntm, ntn, oo, [](int, int) { return true; })) {
        const int i = ij.first, j = ij.second;
        Task t;
        t.ti = i;
        t.tj = j;
        const TileRef c = stored_tile(C, ldc, p.esize, T, i, j, M, N);
        t.m = c.rows;
        t.n = c.cols;
        t.c_host = const_cast<char*>(c.host);
        t.load_c = (beta != 0.0);
        t.alpha_step = alpha;
        t.beta_first = beta;
        for (int kt = 0; kt < ntk; ++kt) {
            StepSpec s;
            s.a = ta ? stored_tile(A, lda, p.esize, T, kt, i, a_rows, a_cols) : stored_tile(A, lda, p.esize, T, i, kt, a_rows, a_cols);
            s.b = tb ? stored_tile(B, ldb, p.esize, T, j, kt, b_rows, b_cols) : stored_tile(B, ldb, p.esize, T, kt, j, b_rows, b_cols);
            s.k = ta ? s.a.rows : s.a.cols;
            t.steps.push_back(s);
            t.flops += 2.0 * t.m * t.n * s.k;
        }
        p.flops += t.flops;
        p.tasks.push_back(std::move(t));
    }
}

// Eq. 1b: C_ij = alpha * sum_k A_ik A_jk^T + beta * C_ij over the tiles of one triangle.
void build_syrk(Problem& p, int dtype, int T, bool lower, bool trans, int N, int K, double alpha,
                const void* A, int64_t lda, double beta, void* C, int64_t ldc, const OrderOpts& oo) {
    // trans = false: op(A) = A (N x K): left operand A_ik as stored, right operand A_jk transposed.
    // trans = true : A is K x N: left operand A_ki transposed, right operand A_kj as stored.
    init_problem(p, dtype, T, trans, !trans, C, ldc, N, N);
    const int nt = cdiv(N, T), ntk = (alpha == 0.0) ? 0 : cdiv(K, T);
    const int64_t a_rows = trans ? K : N, a_cols = trans ? N : K;
    auto keep = [lower](int i, int j) { return lower ? i >= j : i <= j; };
    for (auto ij : superblock_order(nt, nt, oo, keep)) {
        const int i = ij.first, j = ij.second;
        Task t;
        t.ti = i;
        t.tj = j;
        const TileRef c = stored_tile(C, ldc, p.esize, T, i, j, N, N);
        t.m = c.rows;
        t.n = c.cols;
        t.c_host = const_cast<char*>(c.host);
        // A diagonal tile is written back whole, so its other triangle must hold the host's
        // values even when beta == 0 (then the kernel still does not read it).
        t.load_c = (beta != 0.0) || (i == j);
        t.alpha_step = alpha;
        t.beta_first = beta;
        if (i == j) t.c_flags = lower ? TS_C_LOWER : TS_C_UPPER;
        for (int kt = 0; kt < ntk; ++kt) {
            StepSpec s;
            s.a = trans ? stored_tile(A, lda, p.esize, T, kt, i, a_rows, a_cols) : stored_tile(A, lda, p.esize, T, i, kt, a_rows, a_cols);
            s.b = trans ? stored_tile(A, lda, p.esize, T, kt, j, a_rows, a_cols) : stored_tile(A, lda, p.esize, T, j, kt, a_rows, a_cols);
            s.k = trans ? s.a.rows : s.a.cols;
            t.steps.push_back(s);
            t.flops += (i == j ? 1.0 : 2.0) * t.m * t.n * s.k;
        }
        p.flops += t.flops;
        p.tasks.push_back(std::move(t));
    }
}

// Eq. 1e: C_ij = alpha * sum_k A_ik B_jk^T + alpha * sum_k B_ik A_jk^T + beta * C_ij over one triangle:
// two k-steps per k tile, both through the same kernel variant.
void build_syr2k(Problem& p, int dtype, int T, bool lower, bool trans, int N, int K, double alpha,
                 const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                 const OrderOpts& oo) {
    init_problem(p, dtype, T, trans, !trans, C, ldc, N, N);
    p.steps_per_k = 2;
    const int nt = cdiv(N, T), ntk = (alpha == 0.0) ? 0 : cdiv(K, T);
    const int64_t rows = trans ? K : N, cols = trans ? N : K;
    auto keep = [lower](int i, int j) { return lower ? i >= j : i <= j; };
    auto tile_of = [&](const void* X, int64_t ldx, int t, int kt) {
        return trans ? stored_tile(X, ldx, p.esize, T, kt, t, rows, cols) : stored_tile(X, ldx, p.esize, T, t, kt, rows, cols);
    };
    for (auto ij : superblock_order(nt, nt, oo, keep)) {
        const int i = ij.first, j = ij.second;
        Task t;
        t.ti = i;
        t.tj = j;
        const TileRef c = stored_tile(C, ldc, p.esize, T, i, j, N, N);
        t.m = c.rows;
        t.n = c.cols;
        t.c_host = const_cast<char*>(c.host);
        t.load_c = (beta != 0.0) || (i == j);
        t.alpha_step = alpha;
        t.beta_first = beta;
        if (i == j) t.c_flags = lower ? TS_C_LOWER : TS_C_UPPER;
        for (int kt = 0; kt < ntk; ++kt)
            for (int half = 0; half < 2; ++half) {
                StepSpec s;
                s.a = tile_of(half ? B : A, half ? ldb : lda, i, kt);
                s.b = tile_of(half ? A : B, half ? lda : ldb, j, kt);
                s.k = trans ? s.a.rows : s.a.cols;
                t.steps.push_back(s);
                t.flops += (i == j ? 1.0 : 2.0) * t.m * t.n * s.k;
            }
        p.flops += t.flops;
        p.tasks.push_back(std::move(t));
    }
}

// Eq. 1f: C_ij = alpha * sum_k S_ik B_kj + beta * C_ij (left) with S the symmetric matrix whose
// `lower` (or upper) triangle A stores: a tile of S outside the stored triangle is the mirrored
// stored tile transposed, the diagonal tile is the stored one completed by reflection; both are
// made on the device, once, from the stored tile, so every k-step is a plain product.
void build_symm(Problem& p, int dtype, int T, bool left, bool lower, int M, int N, double alpha,
                const void* A, int64_t lda, const void* B, int64_t ldb, double beta, void* C, int64_t ldc,
                const OrderOpts& oo) {
    init_problem(p, dtype, T, false, false, C, ldc, M, N);
    const int ntm = cdiv(M, T), ntn = cdiv(N, T);
    const int na = left ? M : N, nta = (alpha == 0.0) ? 0 : cdiv(na, T);
    for (auto ij : superblock_order(ntm, ntn, oo, [](int, int) { return true; })) {
        const int i = ij.first, j = ij.second;
        Task t;
        t.ti = i;
        t.tj = j;
        const TileRef c = stored_tile(C, ldc, p.esize, T, i, j, M, N);
        t.m = c.rows;
        t.n = c.cols;
        t.c_host = const_cast<char*>(c.host);
        t.load_c = (beta != 0.0);
        t.alpha_step = alpha;
        t.beta_first = beta;
        for (int kt = 0; kt < nta; ++kt) {
            StepSpec s;
            // tile (r, cidx) of S as the product needs it
            const int r = left ? i : kt, cidx = left ? kt : j;
            const bool stored = lower ? (r >= cidx) : (r <= cidx);
            const TileRef st = stored ? stored_tile(A, lda, p.esize, T, r, cidx, na, na) : stored_tile(A, lda, p.esize, T, cidx, r, na, na);
            if (left) {
                s.a = st;
                s.a_mirror = !stored;
                s.b = stored_tile(B, ldb, p.esize, T, kt, j, M, N);
                s.k = s.b.rows;
                if (r == cidx) { s.a_sym = true; s.sym_lower = lower; }
            } else {
                s.a = stored_tile(B, ldb, p.esize, T, i, kt, M, N);
                s.b = st;
                s.b_mirror = !stored;
                s.k = s.a.cols;
                if (r == cidx) { s.b_sym = true; s.sym_lower = lower; }
            }
            t.steps.push_back(s);
            t.flops += 2.0 * t.m * t.n * s.k;
        }
        p.flops += t.flops;
        p.tasks.push_back(std::move(t));
    }
}

// Eq. 1d with alpha on every term: B_ij = alpha * sum_k op(A)_ik B_kj (left) or
// alpha * sum_k B_ik op(A)_kj (right); the sum covers the tiles where op(A) is non-zero and
// the diagonal tile of A is masked to its triangle inside the kernel.
void build_trmm(Problem& p, int dtype, int T, bool left, bool lower, bool trans, bool unit, int M, int N,
                double alpha, const void* A, int64_t lda, void* B, int64_t ldb, const OrderOpts& oo) {
    init_problem(p, dtype, T, left ? trans : false, left ? false : trans, B, ldb, M, N);
    const int ntm = cdiv(M, T), ntn = cdiv(N, T);
    const int na = left ? M : N;                 // order of A
    const bool eff_lower = lower != trans;       // op(A) is lower triangular
    const uint32_t tri = (left ? TS_TRI_A : TS_TRI_B) | (lower ? TS_TRI_LOWER : 0u) | (unit ? TS_TRI_UNIT : 0u);
    (void)oo;
    // One panel = one tile column (left) or tile row (right) of B.
    const int npanels = left ? ntn : ntm, per_panel = left ? ntm : ntn;
    p.panels.resize(npanels);
    for (int pp = 0; pp < npanels; ++pp) {
        Panel& pn = p.panels[pp];
        pn.ntasks = per_panel;
        for (int q = 0; q < per_panel; ++q)
            pn.tiles.push_back(left ? stored_tile(B, ldb, p.esize, T, q, pp, M, N) : stored_tile(B, ldb, p.esize, T, pp, q, M, N));
        for (int q = 0; q < per_panel; ++q) {
            const int i = left ? q : pp, j = left ? pp : q;
            Task t;
            t.ti = i;
            t.tj = j;
            const TileRef c = stored_tile(B, ldb, p.esize, T, i, j, M, N);
            t.m = c.rows;
            t.n = c.cols;
            t.c_host = const_cast<char*>(c.host);
            t.load_c = false;
            t.alpha_step = alpha;
            t.beta_first = 0.0;
            t.panel = pp;
            if (alpha != 0.0) {
                const int d = left ? i : j;      // index of the diagonal tile this task meets
                // left:  k runs over tile columns of op(A) row i   -> k <= i (lower) or k >= i (upper)
                // right: k runs over tile rows of op(A) column j   -> k >= j (lower) or k <= j (upper)
                const bool below = left ? eff_lower : !eff_lower;
                // Step q of every task is the same tile index along k: 0, 1, 2 ... where the tasks' ranges
                // all start at 0, and nt-1, nt-2, ... where they all end at nt-1.  Tasks that advance
                // together (the wide schedule's rounds) then share the tiles of one k, which arrive one k
                // after the other; counted from the diagonal instead, the first round alone would touch
                // every tile of B (measured, N = 12288, wide: 55.4 ms against 40.2 for the mirrored case).
                const int k0 = below ? 0 : d, k1 = below ? d : cdiv(na, T) - 1;
                for (int kq = k0; kq <= k1; ++kq) {
                    const int kt = below ? kq : k1 - (kq - k0);
                    StepSpec s;
                    if (left) {
                        s.a = trans ? stored_tile(A, lda, p.esize, T, kt, i, na, na) : stored_tile(A, lda, p.esize, T, i, kt, na, na);
                        s.b = stored_tile(B, ldb, p.esize, T, kt, j, M, N);
                        s.k = s.b.rows;
                    } else {
                        s.a = stored_tile(B, ldb, p.esize, T, i, kt, M, N);
                        s.b = trans ? stored_tile(A, lda, p.esize, T, j, kt, na, na) : stored_tile(A, lda, p.esize, T, kt, j, na, na);
                        s.k = s.a.cols;
                    }
                    if (kt == d) s.seg_flags = tri;
                    t.steps.push_back(s);
                    t.flops += (kt == d ? 1.0 : 2.0) * t.m * t.n * s.k;
                }
            }
            p.flops += t.flops;
            p.tasks.push_back(std::move(t));
        }
    }
}

// Eq. 1c with alpha placed as the BLAS standard has it:
//   left : X_ij = inv(op(A)_ii) * (alpha B_ij - sum_k op(A)_ik X_kj),  k < i (lower) or k > i (upper)
//   right: X_ij = (alpha B_ij - sum_k X_ik op(A)_kj) * inv(op(A)_jj),  k < j (upper) or k > j (lower)
// X_kj / X_ik are results of other tasks: true dependencies, recorded in StepSpec::dep.  The
// queue is ordered by dependency level so that every task's producers precede it.
void build_trsm(Problem& p, int dtype, int T, bool left, bool lower, bool trans, bool unit, int M, int N,
                double alpha, const void* A, int64_t lda, void* B, int64_t ldb, const OrderOpts& oo) {
    init_problem(p, dtype, T, left ? trans : false, left ? false : trans, B, ldb, M, N);
    p.results_are_operands = true;
    (void)oo;
    const int ntm = cdiv(M, T), ntn = cdiv(N, T);
    const int na = left ? M : N, nta = cdiv(na, T);
    const bool eff_lower = lower != trans;
    // forward: the solve proceeds from tile index 0 upwards along the dependent dimension
    const bool forward = left ? eff_lower : !eff_lower;
    const uint32_t dflags = (lower ? TS_TRI_LOWER : 0u) | (unit ? TS_TRI_UNIT : 0u);
    std::map<std::pair<int, int>, int> index;
    for (int lvl = 0; lvl < nta; ++lvl) {
        const int d = forward ? lvl : nta - 1 - lvl;     // tile index along the dependent dimension
        const int nother = left ? ntn : ntm;
        for (int o = 0; o < nother; ++o) {
            const int i = left ? d : o, j = left ? o : d;
            Task t;
            t.ti = i;
            t.tj = j;
            const TileRef c = stored_tile(B, ldb, p.esize, T, i, j, M, N);
            t.m = c.rows;
            t.n = c.cols;
            t.c_host = const_cast<char*>(c.host);
            t.load_c = true;
            t.alpha_step = -1.0;
            t.beta_first = alpha;
            t.solve = true;
            t.solve_on_right = !left;
            t.diag = stored_tile(A, lda, p.esize, T, d, d, na, na);
            t.diag_flags = dflags;
            for (int q = 0; q < lvl; ++q) {
                const int kt = forward ? q : nta - 1 - q;   // already solved tile indices
                StepSpec s;
                if (left) {
                    s.a = trans ? stored_tile(A, lda, p.esize, T, kt, i, na, na) : stored_tile(A, lda, p.esize, T, i, kt, na, na);
                    s.b = stored_tile(B, ldb, p.esize, T, kt, j, M, N);
                    s.k = s.b.rows;
                    s.b_is_dep = true;
                    s.dep = index[{kt, j}];
                } else {
                    s.a = stored_tile(B, ldb, p.esize, T, i, kt, M, N);
                    s.b = trans ? stored_tile(A, lda, p.esize, T, j, kt, na, na) : stored_tile(A, lda, p.esize, T, kt, j, na, na);
                    s.k = s.a.cols;
                    s.a_is_dep = true;
                    s.dep = index[{i, kt}];
                }
                t.steps.push_back(s);
                t.flops += 2.0 * t.m * t.n * s.k;
            }
            t.flops += 1.0 * t.m * t.n * (left ? t.m : t.n);
            p.flops += t.flops;
            index[{i, j}] = (int)p.tasks.size();
            p.tasks.push_back(std::move(t));
        }
    }
}

}  // namespace blasx
