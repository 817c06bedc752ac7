// Descriptor of one tile step, shared by the host scheduler and the device kernels.
//
// A tile step is the unit of work of the tile algorithms (Section III.B, Eq. 1a-1d):
//     C <- alpha * op(A) * op(B) + beta * C
// (plus, optionally, a second addend tile D) on one m x n output tile with one k-deep pair of operand tiles.  All three tiles
// live in HBM, column-major.  A and B are stored as they are in the host matrix; a
// transposed operand is transposed while it is staged into LDS (Section III.C), never
// in memory.
#pragma once
#include <stdint.h>

namespace blasx {

enum : uint32_t {
    TS_TRANS_A   = 1u << 0,  // op(A) = A^T: A is stored k x m
    TS_TRANS_B   = 1u << 1,  // op(B) = B^T: B is stored n x k
    // Triangular operand (diagonal tiles of TRMM/TRSM, Eq. 1c-1d): only one triangle of the
    // *stored* square tile is real data; the rest is read as zero (and as one on a unit
    // diagonal) without touching memory contents' meaning.
    TS_TRI_A     = 1u << 2,  // the mask applies to A
    TS_TRI_B     = 1u << 3,  // the mask applies to B
    TS_TRI_LOWER = 1u << 4,  // stored lower triangle is the data (else upper)
    TS_TRI_UNIT  = 1u << 5,  // diagonal is taken as one
    // Output triangle (diagonal tiles of SYRK, Eq. 1b): only this triangle of C is read/written.
    TS_C_LOWER   = 1u << 6,
    TS_C_UPPER   = 1u << 7,
    // Every operand tile of the step is stored with zeros between its true extent and the next
    // multiple of the macro-tile edge, in both directions, and that much storage exists: the
    // unpredicated kernel may then run on the padded extents (products with the padding are zero;
    // rows and columns of C beyond m and n are computed and not stored).
    TS_PADDED    = 1u << 8,
};

// One k-deep pair of operand tiles.  Several of them chained in one TileStep are
// summed into the same accumulators before C is touched once.
struct TileSeg {
    const void* A;
    const void* B;
    int32_t  k;              // inner dimension of this pair (> 0)
    uint32_t flags;          // TS_TRI_* of this pair only
};

constexpr int kMaxChain = 8;

// C <- alpha * sum_s op(A_s) op(B_s) + beta * C (+ D) for one output tile.  Extents and leading
// dimensions are at most 8192 (the largest tile edge), so 16 bits hold them and 16 steps with 8
// pairs each fit the kernel-argument segment.
struct TileStep {
    void*       C;
    const void* D;           // optional addend tile (shape and leading dimension of C), or null:
                             // partial sums of earlier launches when C itself arrives late
    TileSeg  seg[kMaxChain];
    double   alpha, beta;    // beta == 0: C is not read
    uint32_t flags;          // TS_TRANS_*, TS_C_*
    uint32_t wg_begin;       // first workgroup (virtual index) of this step within its launch
    uint16_t lda, ldb, ldc;  // leading dimensions in elements (same for every pair)
    uint16_t m, n;           // C is m x n
    uint16_t nseg;           // 0: C <- beta * C (+ D) only
};
static_assert(sizeof(TileStep) == 248, "tile step layout");

// Up to this many tile steps travel by value in the kernel arguments of one launch
// (the whole pack must stay below the 4 KB kernel-argument limit).
constexpr int kMaxStepsPerLaunch = 16;

struct LaunchPack {
    int32_t  nsteps;
    uint32_t total_wg;       // sum over steps of macro_tiles()
    TileStep step[kMaxStepsPerLaunch];
};
static_assert(sizeof(LaunchPack) <= 4096, "launch pack must fit the kernel-argument segment");

constexpr int kBM = 128;     // macro-tile rows of C per workgroup
constexpr int kBN = 128;     // macro-tile columns of C per workgroup
constexpr int kBK = 16;      // depth of one LDS slab

// Workgroups of a step: one per macro-tile of C; with an output triangle (TS_C_LOWER / TS_C_UPPER, the diagonal tiles
// of SYRK and SYR2K) only the macro-tiles that touch the triangle, column by column (tile_steps_kernel maps its
// workgroup index the same way).
inline uint32_t macro_tiles(int m, int n, uint32_t flags = 0) {
    const uint32_t tm = (uint32_t)((m + kBM - 1) / kBM), tn = (uint32_t)((n + kBN - 1) / kBN);
    if (!(flags & (TS_C_LOWER | TS_C_UPPER))) return tm * tn;
    uint32_t count = 0;
    for (uint32_t j = 0; j < tn; ++j) count += (flags & TS_C_LOWER) ? (tm > j ? tm - j : 0) : (j + 1 < tm ? j + 1 : tm);
    return count;
}

// True when a step can run in the unpredicated kernel: whole macro-tiles, every k a multiple of
// two slabs (a slab is 8 sixteen-byte chunks deep: 16 k in fp64, 32 k in fp32; the kernel works on
// slab pairs), operands 16-byte aligned with leading dimensions that keep columns aligned.  Masks are
// fine: operand masks are applied to fragments, the output-triangle mask in the epilogue.  A step of
// zero-padded tiles (TS_PADDED) may have any extents that, rounded up, still lie inside the tiles'
// storage (a square of the leading dimension).
inline int round_up_to(int x, int q) { return (x + q - 1) / q * q; }
inline bool step_is_ragged(const TileStep& st, int dtype) {
    const int epc = dtype == 0 ? 2 : 4;
    if (st.m % kBM || st.n % kBN) return true;
    for (int s = 0; s < st.nseg; ++s)
        if (st.seg[s].k % (16 * epc)) return true;
    return false;
}
inline bool step_is_fast(const TileStep& st, int dtype) {
    const int epc = dtype == 0 ? 2 : 4;          // elements per 16-byte chunk
    const bool padded = st.flags & TS_PADDED;
    if (st.m <= 0 || st.n <= 0 || st.lda % epc || st.ldb % epc) return false;
    if (!padded && (st.m % kBM || st.n % kBN)) return false;
    if (st.flags & ~(TS_TRANS_A | TS_TRANS_B | TS_C_LOWER | TS_C_UPPER | TS_PADDED)) return false;
    if (padded && (round_up_to(st.m, kBM) > st.lda || round_up_to(st.n, kBN) > st.ldb)) return false;
    for (int s = 0; s < st.nseg; ++s) {
        const TileSeg& sg = st.seg[s];
        if (sg.k <= 0) return false;
        if (!padded && sg.k % (16 * epc)) return false;
        if (padded && (round_up_to(sg.k, 16 * epc) > st.lda || round_up_to(sg.k, 16 * epc) > st.ldb)) return false;
        if ((reinterpret_cast<uintptr_t>(sg.A) | reinterpret_cast<uintptr_t>(sg.B)) % 16) return false;
    }
    return true;
}

// Which kernel instantiation a step needs: 0 = fast, 1 = fast with operand masks, 2 = general.
inline int step_mode(const TileStep& st, int dtype) {
    if (!step_is_fast(st, dtype)) return 2;
    for (int s = 0; s < st.nseg; ++s)
        if (st.seg[s].flags) return 1;
    return 0;
}

}  // namespace blasx
