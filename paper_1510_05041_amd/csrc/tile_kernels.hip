// Tile-step kernels for CDNA4 (gfx950): C <- alpha * sum_s op(A_s) * op(B_s) + beta * C (+ D) on
// HBM-resident tiles (Section III.B, Eq. 1a-1f; the call the paper's Alg. 1 makes once per
// (i, j, k), here with up to eight chained k-steps per call; D is an optional second addend
// tile, the partial sums of earlier launches when the host tile of C itself arrives late).
//
// One launch executes a *pack* of tile steps (different output tiles), so that a launch fills
// the 256 CUs even though a single 1024^3 step only has 64 macro-tiles.  The paper shares the
// GPU between 4 tasks by running 4 vendor-BLAS calls on 4 streams; here the sharing happens
// inside one grid instead.
//
// Common to both paths
//   macro-tile = 128 x 128 of C per workgroup
//   MFMA       = v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32, issued on the transposed
//                product (a := B fragment, b := A fragment) so that the 16 lanes that share an
//                accumulator register hold 16 consecutive rows of C: stores to column-major C
//                are 128-byte (fp64) contiguous runs.
//   transposes = never in memory (Section III.C: the stored tile is fetched as it is and
//                transposed on its way through LDS).
//   XCD mapping= hardware deals consecutive workgroup ids round-robin to the 8 XCDs; the
//                virtual index gives each XCD a contiguous range of macro-tiles, i.e. whole
//                steps, so the 64 macro-tiles that share one A and one B tile run under one L2.
//
// General path (macro_tile): any extents, alignment and masks.  256 threads = 4 waves (2 x 2) of
//   64 x 64; k slabs of 16 are fetched into registers with bounds and triangle predicates and
//   stored to a double-buffered LDS layout [k][mn] whose mn index is XOR-swizzled by
//   2*((k>>1)&7), so that both the direct and the transposing stores are conflict-free.
// Fast path (macro_tile_fast): see the comment above it.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

#include "tile_step.h"

namespace blasx {

constexpr int BM = kBM;
constexpr int BN = kBN;
constexpr int BK = kBK;
constexpr int NTHREADS = 256;
constexpr int NXCD = 8;

template <typename T> struct Mfma;

template <> struct Mfma<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    typedef double vec2_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    // accumulator register r of a lane in 16-lane group g holds result row 4*r + g
    static __device__ __forceinline__ int drow(int r, int g) { return 4 * r + g; }
};

template <> struct Mfma<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    typedef float vec2_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    // accumulator register r of a lane in 16-lane group g holds result row 4*g + r
    static __device__ __forceinline__ int drow(int r, int g) { return 4 * g + r; }
};

__device__ __forceinline__ int swz(int l) { return ((l >> 1) & 7) << 1; }

// Value of element (r, c) of a stored square tile under a triangular mask.
template <typename T>
__device__ __forceinline__ T tri_value(const T* p, int ld, int r, int c, uint32_t flags) {
    if (r == c) return (flags & TS_TRI_UNIT) ? T(1) : p[(size_t)r + (size_t)c * ld];
    const bool inside = (flags & TS_TRI_LOWER) ? (r > c) : (r < c);
    return inside ? p[(size_t)r + (size_t)c * ld] : T(0);
}

// One operand slab (16 deep, 128 wide) from HBM into registers, with bounds (mn < mn_valid,
// l < k_valid; out of range reads as zero) and the optional triangular mask.
//   KCONTIG = false: element (mn, l) is at p[mn + l*ld]  (A not transposed, B transposed)
//   KCONTIG = true : element (mn, l) is at p[l + mn*ld]  (A transposed, B not transposed)
template <typename T, bool KCONTIG>
__device__ __forceinline__ void slab_load(typename Mfma<T>::vec2_t (&reg)[4], const T* __restrict__ p, int ld,
                                          int mn_base, int k0, int mn_valid, int k_valid, bool tri,
                                          uint32_t flags, int tid) {
    typedef typename Mfma<T>::vec2_t V2;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        V2 v = {T(0), T(0)};
        if (!KCONTIG) {
            const int mn = mn_base + (tid & 63) * 2;
            const int l = k0 + (tid >> 6) + 4 * q;
            if (l < k_valid) {
                if (tri) {
                    if (mn < mn_valid) v.x = tri_value(p, ld, mn, l, flags);
                    if (mn + 1 < mn_valid) v.y = tri_value(p, ld, mn + 1, l, flags);
                } else {
                    if (mn < mn_valid) v.x = p[(size_t)mn + (size_t)l * ld];
                    if (mn + 1 < mn_valid) v.y = p[(size_t)mn + 1 + (size_t)l * ld];
                }
            }
        } else {
            const int l = k0 + (tid & 7) * 2;
            const int mn = mn_base + (tid >> 3) + 32 * q;
            if (mn < mn_valid) {
                if (tri) {
                    if (l < k_valid) v.x = tri_value(p, ld, l, mn, flags);
                    if (l + 1 < k_valid) v.y = tri_value(p, ld, l + 1, mn, flags);
                } else {
                    if (l < k_valid) v.x = p[(size_t)l + (size_t)mn * ld];
                    if (l + 1 < k_valid) v.y = p[(size_t)l + 1 + (size_t)mn * ld];
                }
            }
        }
        reg[q] = v;
    }
}

// Registers into one operand's LDS slab ([BK][128], swizzled).
template <typename T, bool KCONTIG>
__device__ __forceinline__ void slab_store(T* __restrict__ lds, const typename Mfma<T>::vec2_t (&reg)[4], int tid) {
    typedef typename Mfma<T>::vec2_t V2;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (!KCONTIG) {
            const int mn = (tid & 63) * 2;
            const int l = (tid >> 6) + 4 * q;
            *reinterpret_cast<V2*>(lds + l * 128 + (mn ^ swz(l))) = reg[q];
        } else {
            const int l = (tid & 7) * 2;
            const int mn = (tid >> 3) + 32 * q;
            const int col = mn ^ swz(l);
            lds[l * 128 + col] = reg[q].x;
            lds[(l + 1) * 128 + col] = reg[q].y;
        }
    }
}

// General path: one 128 x 128 macro-tile of one step, any extents and masks.
template <typename T, bool TA, bool TB>
__device__ __forceinline__ void macro_tile(const TileStep& st, int i_base, int j_base) {
    typedef typename Mfma<T>::acc_t acc_t;
    typedef typename Mfma<T>::vec2_t V2;
    // [buffer][operand][k][mn]; always addressed through this array so that every access is a
    // ds_ instruction (LDS address space known to the compiler).
    __shared__ __attribute__((aligned(16))) T lds[4 * BK * 128];
    constexpr int OPERAND = BK * 128, BUFFER = 2 * BK * 128;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r16 = lane & 15;
    const int wm = wave & 1, wn = wave >> 1;

    T* __restrict__ C = static_cast<T*>(st.C);
    const int m = st.m, n = st.n;
    const int lda = st.lda, ldb = st.ldb;
    const int nseg = st.nseg;

    acc_t acc[4][4];
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < 4; ++bj) acc[bi][bj] = acc_t{0, 0, 0, 0};

    // Fragment read offsets: k row l = 4*kk + g, column (r16 ^ swz(l)) = (r16 ^ 2*(g>>1)) ^ 4*kk.
    const int frag_col = r16 ^ ((g >> 1) << 1);
    const int fragA = g * 128 + wm * 64, fragB = OPERAND + g * 128 + wn * 64;

    // Prefetch cursor: pair `pseg`, slab `pslab` of it is the next one to fetch from HBM.  The
    // slab loop runs across the chained pairs without draining the pipeline in between.
    int pseg = 0, pslab = 0;
    int pk = nseg > 0 ? st.seg[0].k : 0;
    uint32_t pflags = nseg > 0 ? st.seg[0].flags : 0;
    const T* A = nseg > 0 ? static_cast<const T*>(st.seg[0].A) : nullptr;
    const T* B = nseg > 0 ? static_cast<const T*>(st.seg[0].B) : nullptr;

    V2 ra[4], rb[4];
    bool more = nseg > 0;
    if (more) {
        slab_load<T, TA>(ra, A, lda, i_base, 0, m, pk, pflags & TS_TRI_A, pflags, tid);
        slab_load<T, !TB>(rb, B, ldb, j_base, 0, n, pk, pflags & TS_TRI_B, pflags, tid);
        slab_store<T, TA>(lds, ra, tid);
        slab_store<T, !TB>(lds + OPERAND, rb, tid);
    }
    __syncthreads();

    int cur = 0;
    while (more) {
        // advance the prefetch cursor to the slab after the one now in LDS
        ++pslab;
        if (pslab * BK >= pk) {
            ++pseg;
            pslab = 0;
            more = pseg < nseg;
            if (more) {
                pk = st.seg[pseg].k;
                pflags = st.seg[pseg].flags;
                A = static_cast<const T*>(st.seg[pseg].A);
                B = static_cast<const T*>(st.seg[pseg].B);
            }
        }
        if (more) {
            slab_load<T, TA>(ra, A, lda, i_base, pslab * BK, m, pk, pflags & TS_TRI_A, pflags, tid);
            slab_load<T, !TB>(rb, B, ldb, j_base, pslab * BK, n, pk, pflags & TS_TRI_B, pflags, tid);
        }
        // Fragments are double buffered: those of sub-step kk+1 are requested before the MFMAs of kk.
        T fa[2][4], fb[2][4];
#pragma unroll
        for (int bi = 0; bi < 4; ++bi) fa[0][bi] = lds[cur + fragA + bi * 16 + frag_col];
#pragma unroll
        for (int bj = 0; bj < 4; ++bj) fb[0][bj] = lds[cur + fragB + bj * 16 + frag_col];
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            const int c = kk & 1, nx = c ^ 1;
            if (kk + 1 < BK / 4) {
                const int col = frag_col ^ (4 * (kk + 1));
#pragma unroll
                for (int bi = 0; bi < 4; ++bi) fa[nx][bi] = lds[cur + fragA + (kk + 1) * 4 * 128 + bi * 16 + col];
#pragma unroll
                for (int bj = 0; bj < 4; ++bj) fb[nx][bj] = lds[cur + fragB + (kk + 1) * 4 * 128 + bj * 16 + col];
            }
#pragma unroll
            for (int bi = 0; bi < 4; ++bi)
#pragma unroll
                for (int bj = 0; bj < 4; ++bj) acc[bi][bj] = Mfma<T>::run(fb[c][bj], fa[c][bi], acc[bi][bj]);
        }
        if (more) {
            slab_store<T, TA>(lds + (cur ^ BUFFER), ra, tid);
            slab_store<T, !TB>(lds + (cur ^ BUFFER) + OPERAND, rb, tid);
        }
        __syncthreads();
        cur ^= BUFFER;
    }

    const uint32_t flags = st.flags;
    const T alpha = (T)st.alpha, beta = (T)st.beta;
    const bool use_c = (st.beta != 0.0);
    const T* __restrict__ D = static_cast<const T*>(st.D);
    const int ldc = st.ldc;
#pragma unroll
    for (int bj = 0; bj < 4; ++bj)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = j_base + wn * 64 + bj * 16 + Mfma<T>::drow(r, g);
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                const int i = i_base + wm * 64 + bi * 16 + r16;
                if (i >= m || j >= n) continue;
                if ((flags & TS_C_LOWER) && i < j) continue;
                if ((flags & TS_C_UPPER) && i > j) continue;
                T* p = C + (size_t)i + (size_t)j * ldc;
                T v = alpha * acc[bi][bj][r];
                if (use_c) v += beta * (*p);
                if (D) v += D[(size_t)i + (size_t)j * ldc];
                *p = v;
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Fast path: operand slabs go from HBM straight into LDS (global_load_lds_dwordx4), with no
// staging registers and no LDS store instructions, two stages deep.
//
// A 16-byte chunk (EPC = 2 doubles or 4 floats) is the unit of both the copy and the layout; a
// slab is 8 chunks deep (16 k in fp64, 32 k in fp32) and 128 wide, 16 KB per operand.  Lane L of a
// wave-wide copy always lands at chunk L of the 1 KB window the instruction names, but WHICH 16
// bytes of the operand a lane fetches is free, and that choice makes the layout:
//   mn-contiguous source (A not transposed / B transposed): plain [k][128] rows; an instruction
//     copies one (fp64) or two (fp32) whole k rows, contiguous in HBM; a fragment is a read of 16
//     consecutive elements.
//   k-contiguous source (A transposed / B not transposed): chunk (mn, q) = k = EPC*q .. EPC*q+EPC-1
//     of column mn at chunk index mn*8 + (q ^ (mn & 7)); an instruction copies 8 columns x 128
//     contiguous bytes; a fragment read yields EPC consecutive k values, and the XOR spreads the 16
//     lanes of a fragment read over all banks.
// MFMA group (c, h) consumes k = 4*EPC*c + EPC*g + h in lane group g (c: half of the slab, h:
// position in the chunk), the same assignment for both operands, so either layout pairs with
// either and the four transpose variants run at the same speed.
//
// Shape, double precision: 512 threads = 8 waves (2 x 4) per workgroup, each wave owning 64 x 32 of the
// macro-tile (4 x 2 MFMA blocks, 64 accumulator registers), two workgroups per CU = 4 waves per SIMD to
// cover barrier and LDS latencies.
// Shape, single precision: 256 threads = 4 waves (2 x 2), each wave owning 64 x 64 (4 x 4 blocks, again 64
// accumulator registers), two workgroups per CU = 2 waves per SIMD.  A single-precision MFMA takes half the
// cycles of a double-precision one for the same two operand registers, so with the 64 x 32 shape a wave
// had to fetch its operands from LDS twice as often per MFMA cycle (the MFMA pipes were busy 87.6 % of the
// time against 94 % in double precision); the square 64 x 64 wave tile needs a third fewer operand reads
// per flop and gives groups of 16 MFMAs (512 cycles) per block row instead of 8 (256 cycles).
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

template <typename T> struct FastShape {
    static constexpr int EPC = 16 / (int)sizeof(T);      // elements per 16-byte chunk
    static constexpr int SLAB_K = 8 * EPC;               // k depth of one slab
    static constexpr int ROWS_PER_COPY = 1024 / (128 * (int)sizeof(T));   // k rows one wave-wide copy covers
    static constexpr int LANES_PER_ROW = 64 / ROWS_PER_COPY;
    static constexpr int STAGE = 128 * SLAB_K;           // elements per operand stage (16 KB)
    static constexpr int WAVES_N = sizeof(T) == 8 ? 4 : 2;   // waves form a 2 x WAVES_N grid over the macro-tile
    static constexpr int NBJ = 128 / (16 * WAVES_N);     // 16-column MFMA blocks per wave: 2 or 4 (rows: always 4)
    static constexpr int WAVE_N = 16 * NBJ;              // columns of C per wave
    static constexpr int WAVES = 2 * WAVES_N;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int DMA_PER_WAVE = 16 / WAVES;      // wave-wide copies per operand slab and wave
    // When a slab's copies are issued: copy i of each operand goes out at position i / COPY_PP - 1, where -1 is
    // right after the barrier that frees the stage and u >= 0 is together with unit u of the next slab.
    // Measured: one copy per operand and position in fp64 (2 positions), two in fp32 (2 positions); all of a slab's
    // copies in one burst after the barrier is 0.5 % slower in both, one per unit in fp32 1 % slower.
    static constexpr int COPY_PP = sizeof(T) == 8 ? 1 : DMA_PER_WAVE / 2;
};

// Source of this lane for the first of its wave's copies of an operand slab, as an element offset from
// the tile's first element.
template <typename T, bool KCONTIG>
__device__ __forceinline__ size_t dma_offset(int ld, int mn_base, int wave, int lane) {
    typedef FastShape<T> S;
    if (!KCONTIG) {
        const int row = wave * S::DMA_PER_WAVE * S::ROWS_PER_COPY + lane / S::LANES_PER_ROW;
        // fp32: a 4-byte fragment read serves 32 lanes per pass = two lane groups g, whose rows are
        // 4 apart and would start at the same bank; every other group of 4 rows is therefore stored
        // with its columns shifted by half the banks (col ^ 16), i.e. chunk ^ 4.  The two rows of one
        // copy fall in the same group of 4; a wave's later copies may fall in the other one (dma_alt).
        const int chunk = (lane % S::LANES_PER_ROW) ^ (sizeof(T) == 4 ? 4 * ((row >> 2) & 1) : 0);
        return (size_t)(mn_base + chunk * S::EPC) + (size_t)row * ld;
    }
    const int m = lane >> 3, q = (lane & 7) ^ m;
    return (size_t)(S::EPC * q) + (size_t)(mn_base + wave * S::DMA_PER_WAVE * 8 + m) * ld;
}
// What to add (in elements) to this lane's source address for a copy whose rows lie in the other kind
// of 4-row group than the wave's first copy (mn-contiguous fp32 sources only, else 0): chunk ^ 4.
template <typename T, bool KCONTIG>
__device__ __forceinline__ int dma_alt(int wave, int lane) {
    typedef FastShape<T> S;
    if (KCONTIG || sizeof(T) != 4) return 0;
    const int row = wave * S::DMA_PER_WAVE * S::ROWS_PER_COPY + lane / S::LANES_PER_ROW;
    const int chunk = (lane % S::LANES_PER_ROW) ^ (4 * ((row >> 2) & 1));
    return (chunk & 4) ? -4 * S::EPC : 4 * S::EPC;
}

// The lane-dependent part of a copy's source address, as a byte offset from the first element of the tile's
// current slab; worked out once per macro-tile.  The rest of the address (tile, slab, copy number) is the same
// for the whole wave and stays in scalar registers (a buffer descriptor for the tile and a scalar byte offset):
// a copy then reads one 32-bit address register per lane instead of a 64-bit pair, and neither a copy nor the
// move to the next slab costs a vector instruction.
// off[1]: for the copies whose rows lie in the other kind of 4-row group (see dma_alt).
template <typename T, bool KCONTIG> struct CopyLane {
    uint32_t off[2];
    __device__ __forceinline__ CopyLane(int ld, int mn_base, int wave, int lane) {
        off[0] = (uint32_t)(dma_offset<T, KCONTIG>(ld, mn_base, wave, lane) * sizeof(T));
        off[1] = off[0] + (uint32_t)(dma_alt<T, KCONTIG>(wave, lane) * (int)sizeof(T));
    }
};

// Raw buffer descriptor over a tile (no stride, no swizzle, 32-bit data format); the range is left at its
// maximum: the host has checked the steps of a fast-path pack against the tile extents.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* tile) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(tile), 0, 0x7fffffff, 0x27000);
}

// Copy number i (0 .. DMA_PER_WAVE - 1) of this wave's share of one operand slab, from the slab that starts
// `slab_off` bytes into the tile, into the operand's 16 KB LDS window `stage`: lane l's 16 bytes land at byte
// 16 l of the copy's 1 KB part of it.
template <typename T, bool KCONTIG>
__device__ __forceinline__ void dma_piece(__amdgpu_buffer_rsrc_t tile, uint32_t slab_off, int ld, const CopyLane<T, KCONTIG>& cl,
                                          T* stage, int wave, int i) {
    typedef FastShape<T> S;
    // a wave's copies start at a multiple of 8 rows, so which 4-row group copy i falls in depends on i alone
    static_assert(sizeof(T) != 4 || (S::DMA_PER_WAVE * S::ROWS_PER_COPY) % 8 == 0, "copy rows per wave");
    const bool other = !KCONTIG && sizeof(T) == 4 && (((S::ROWS_PER_COPY * i) >> 2) & 1);
    const uint32_t rows = slab_off + (uint32_t)((KCONTIG ? 8 * i : S::ROWS_PER_COPY * i) * ld * (int)sizeof(T));
    T* dst = stage + (wave * S::DMA_PER_WAVE + i) * (1024 / (int)sizeof(T));
    __builtin_amdgcn_raw_ptr_buffer_load_lds(tile, (lds_ptr_t)dst, 16, (int)cl.off[other], (int)rows, 0, 0);
}
// All of them at once.
template <typename T, bool KCONTIG>
__device__ __forceinline__ void dma_slab(__amdgpu_buffer_rsrc_t tile, uint32_t slab_off, int ld, const CopyLane<T, KCONTIG>& cl, T* stage, int wave) {
#pragma unroll
    for (int i = 0; i < FastShape<T>::DMA_PER_WAVE; ++i) dma_piece<T, KCONTIG>(tile, slab_off, ld, cl, stage, wave, i);
}

// Where a lane finds its operand values in an operand's LDS stage: the lane-dependent part of the element
// index, worked out once per macro-tile; everything else (block b, half slab c, position h) is a constant of
// the instruction.  `base` = first row / column of the wave's part of the macro-tile.
//   mn-contiguous layout: element (k, mn) at k * 128 + (mn ^ swz(k)); fp32 rows of odd 4-row groups have their
//     columns shifted by 16 (swz = 16 for lane groups g = 1, 3): mn ^ 16 is mn + 16 for even blocks b and mn - 16
//     for odd ones, hence two bases.
//   k-contiguous layout: chunk (mn, q) at mn * 8 + (q ^ (mn & 7)), q = 4 c + g: the chunk index of c = 1 is that
//     of c = 0 with bit 2 flipped, hence two bases again.
template <typename T, bool KCONTIG> struct LaneBase {
    int v[2];
    __device__ __forceinline__ LaneBase(int base, int g, int r16) {
        typedef FastShape<T> S;
        if (!KCONTIG) {
            const int sh = sizeof(T) == 4 ? 16 * (g & 1) : 0;
            v[0] = S::EPC * g * 128 + base + r16 + sh;       // even blocks
            v[1] = S::EPC * g * 128 + base + r16 - sh;       // odd blocks
        } else {
            const int q0 = g ^ (r16 & 7);
            v[0] = ((base + r16) * 8 + q0) * S::EPC;          // c = 0
            v[1] = ((base + r16) * 8 + (q0 ^ 4)) * S::EPC;    // c = 1
        }
    }
    // element index of position h (k = 4 EPC c + EPC g + h) of block b
    __device__ __forceinline__ int at(int b, int c, int h) const {
        typedef FastShape<T> S;
        if (!KCONTIG) return v[b & 1] + (4 * S::EPC * c + h) * 128 + b * 16;
        return v[c] + b * 128 * S::EPC + h;
    }
};

// Element (r, c) of a stored triangular tile, given the value v that memory holds there.
template <typename T>
__device__ __forceinline__ T tri_select(T v, int r, int c, uint32_t flags) {
    if (r == c) return (flags & TS_TRI_UNIT) ? T(1) : v;
    const bool inside = (flags & TS_TRI_LOWER) ? (r > c) : (r < c);
    return inside ? v : T(0);
}

// Waits for this wave's outstanding LDS reads and pins the wait in place.  The software pipelines
// below request the fragments of step t+1, issue the MFMAs of step t, and only then wait: left
// alone, the compiler sinks every LDS read to just before its first use, or waits for all reads
// right after requesting the next ones, and the wave sits out the LDS latency once per step.
__device__ __forceinline__ void lds_fence() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), other counters untouched
    __builtin_amdgcn_sched_barrier(0);
}

// The MFMAs of a slab are issued in units, and the unit is the stage of a software pipeline that runs
// across the slabs of a macro-tile without ever draining: while the MFMAs of unit u are being issued the
// operand values of unit u + 1 are on their way from LDS to registers -- also when u is the last unit
// of its slab, in which case u + 1 is the first unit of the next slab, read from the other stage right
// after the barrier that says the stage is complete (see macro_tile_fast).
//   double precision: a unit is one MFMA group (c, h), k = 8 c + 2 g + h: 4 values of A, NBJ of B,
//     4 x NBJ MFMAs of 64 cycles; 4 units per slab; the values are double buffered by unit parity.
//   single precision: a unit is (c, block row bi): the 4 values h = 0..3 of A for that block row (one
//     16-byte chunk when A is k-contiguous: conflict-free thanks to the XOR in the layout, where four
//     separate 4-byte reads would collide four ways) and 4 x NBJ MFMAs of 32 cycles against the B values of
//     half-slab c (NBJ chunks, requested together with the A values of unit 0 for c = 0 and of unit 2 for
//     c = 1); 8 units per slab; A double buffered by parity, B by c.
// MASK: one operand of the chained pair is a diagonal tile of a triangular matrix (sflags says which and
// how); its values are masked in registers just before the MFMAs use them, so what the other triangle
// holds in memory never reaches an MFMA.  k0 = k offset of the unit's slab in its pair.
template <typename T> struct FastRegs;
template <> struct FastRegs<double> {
    static constexpr int NU = 4;                               // units per slab
    double a[2][4], b[2][FastShape<double>::NBJ];
};
template <> struct FastRegs<float> {
    static constexpr int NU = 8;
    float a[2][4], b[2][FastShape<float>::NBJ][4];
};

// Requests the operand values of unit u of the slab in (sa, sb).
template <typename T, bool TA, bool TB>
__device__ __forceinline__ void unit_load(FastRegs<T>& R, const T* sa, const T* sb, int u, const LaneBase<T, TA>& la,
                                          const LaneBase<T, !TB>& lb) {
    typedef FastShape<T> S;
    constexpr int NBJ = S::NBJ;
    if constexpr (sizeof(T) == 8) {
        // mn-contiguous operands only: a k-contiguous one comes a whole 16-byte chunk (both h) at a time, see unit_load_late
        const int c = u / S::EPC, h = u % S::EPC;
        if (!TA) {
#pragma unroll
            for (int b = 0; b < 4; ++b) R.a[u & 1][b] = sa[la.at(b, c, h)];
        }
        if (TB) {
#pragma unroll
            for (int b = 0; b < NBJ; ++b) R.b[u & 1][b] = sb[lb.at(b, c, h)];
        }
    } else {
        const int c = u >> 2, bi = u & 3;
        if (TA) {
            const float4 x = *reinterpret_cast<const float4*>(sa + la.at(bi, c, 0));
            R.a[u & 1][0] = x.x; R.a[u & 1][1] = x.y; R.a[u & 1][2] = x.z; R.a[u & 1][3] = x.w;
        } else {
#pragma unroll
            for (int h = 0; h < 4; ++h) R.a[u & 1][h] = sa[la.at(bi, c, h)];
        }
        // the B values of half slab 0 come with unit 0, those of half slab 1 with unit 2 (two units early)
        if (u == 0 || u == 2) {
            const int cb = u >> 1;
#pragma unroll
            for (int b = 0; b < NBJ; ++b) {
                if (!TB) {
                    const float4 x = *reinterpret_cast<const float4*>(sb + lb.at(b, cb, 0));
                    R.b[cb][b][0] = x.x; R.b[cb][b][1] = x.y; R.b[cb][b][2] = x.z; R.b[cb][b][3] = x.w;
                } else {
#pragma unroll
                    for (int h = 0; h < 4; ++h) R.b[cb][b][h] = sb[lb.at(b, cb, h)];
                }
            }
        }
    }
}

// Double precision, k-contiguous operands: the two values h = 0, 1 that a lane needs from half slab c are the two
// halves of one 16-byte chunk, and only a 16-byte read of that layout is free of bank conflicts (eight lanes per
// cycle, eight bank groups; 8-byte reads serve sixteen lanes per cycle and collide in pairs).  So the chunk is read
// whole, into the registers of both units (c, 0) and (c, 1) -- which is only possible once the MFMAs of the unit
// before, (c - 1, 1), have been issued: these requests follow them instead of preceding them.
template <typename T, bool TA, bool TB>
__device__ __forceinline__ void unit_load_late(FastRegs<T>& R, const T* sa, const T* sb, int c, const LaneBase<T, TA>& la,
                                               const LaneBase<T, !TB>& lb) {
    if constexpr (sizeof(T) == 8) {
        typedef typename Mfma<T>::vec2_t V2;
        if (TA) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const V2 x = *reinterpret_cast<const V2*>(sa + la.at(b, c, 0));
                R.a[0][b] = x.x;
                R.a[1][b] = x.y;
            }
        }
        if (!TB) {
#pragma unroll
            for (int b = 0; b < FastShape<T>::NBJ; ++b) {
                const V2 x = *reinterpret_cast<const V2*>(sb + lb.at(b, c, 0));
                R.b[0][b] = x.x;
                R.b[1][b] = x.y;
            }
        }
    }
}

// Masks (MASK) and multiplies unit u; its values must have arrived.
template <typename T, bool TA, bool TB, bool MASK>
__device__ __forceinline__ void unit_mfma(typename Mfma<T>::acc_t (&acc)[4][FastShape<T>::NBJ], FastRegs<T>& R, int u,
                                          int wm, int wn, int g, int r16, uint32_t sflags, int k0, int i_base, int j_base) {
    typedef FastShape<T> S;
    constexpr int NBJ = S::NBJ;
    if constexpr (sizeof(T) == 8) {
        const int c = u / S::EPC, h = u % S::EPC, cur = u & 1;
        if (MASK) {
            const int kg = k0 + 4 * S::EPC * c + S::EPC * g + h;
            if (sflags & TS_TRI_A) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int i = i_base + wm * 64 + b * 16 + r16;
                    R.a[cur][b] = TA ? tri_select(R.a[cur][b], kg, i, sflags) : tri_select(R.a[cur][b], i, kg, sflags);
                }
            }
            if (sflags & TS_TRI_B) {
#pragma unroll
                for (int b = 0; b < NBJ; ++b) {
                    const int j = j_base + wn * S::WAVE_N + b * 16 + r16;
                    R.b[cur][b] = TB ? tri_select(R.b[cur][b], j, kg, sflags) : tri_select(R.b[cur][b], kg, j, sflags);
                }
            }
        }
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int bj = 0; bj < NBJ; ++bj) acc[bi][bj] = Mfma<T>::run(R.b[cur][bj], R.a[cur][bi], acc[bi][bj]);
    } else {
        const int c = u >> 2, bi = u & 3, cur = u & 1;
        if (MASK) {
            if (sflags & TS_TRI_A) {
                const int i = i_base + wm * 64 + bi * 16 + r16;
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const int kg = k0 + 16 * c + 4 * g + h;
                    R.a[cur][h] = TA ? tri_select(R.a[cur][h], kg, i, sflags) : tri_select(R.a[cur][h], i, kg, sflags);
                }
            }
            if ((sflags & TS_TRI_B) && bi == 0) {      // once per half slab, when its first unit is up
#pragma unroll
                for (int b = 0; b < NBJ; ++b) {
                    const int j = j_base + wn * S::WAVE_N + b * 16 + r16;
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const int kg = k0 + 16 * c + 4 * g + h;
                        R.b[c][b][h] = TB ? tri_select(R.b[c][b][h], j, kg, sflags) : tri_select(R.b[c][b][h], kg, j, sflags);
                    }
                }
            }
        }
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
            for (int bj = 0; bj < NBJ; ++bj) acc[bi][bj] = Mfma<T>::run(R.b[c][bj][h], R.a[cur][h], acc[bi][bj]);
    }
}

// The k range [kb, ke) of a chained pair in which the macro-tile at (i_base, j_base) can meet the
// stored triangle of the pair's triangular operand; outside it every product is zero, so those
// slabs are neither copied nor multiplied (half the work of a diagonal tile on average).  Macro-
// tile origins and extents are multiples of two slabs, so the range is a whole number of slab
// pairs.  Element (r, c) of the stored tile is inside a lower triangle when r >= c.
template <bool TA, bool TB>
__device__ __forceinline__ void masked_k_range(uint32_t sflags, int k, int i_base, int j_base, int& kb, int& ke) {
    kb = 0;
    ke = k;
    const bool lower = sflags & TS_TRI_LOWER;
    if (sflags & TS_TRI_A) {
        // op(A)(i, kk) is stored at (kk, i) when transposed, else at (i, kk)
        if (lower != TA) ke = min(ke, i_base + BM);      // needs kk <= i
        else kb = max(kb, i_base);                       // needs kk >= i
    }
    if (sflags & TS_TRI_B) {
        // op(B)(kk, j) is stored at (j, kk) when transposed, else at (kk, j)
        if (lower != TB) kb = max(kb, j_base);           // needs kk >= j
        else ke = min(ke, j_base + BN);                  // needs kk <= j
    }
    if (ke < kb) ke = kb;
}

// Whether the slab k0 .. k0 + slab_k - 1 of a masked pair lies wholly inside the stored triangle
// (diagonal excluded) for every row and column of the macro-tile: such a slab needs no masking.
template <bool TA, bool TB>
__device__ __forceinline__ bool slab_inside_triangle(uint32_t sflags, int k0, int slab_k, int i_base, int j_base) {
    const bool lower = sflags & TS_TRI_LOWER;
    bool inside = true;
    if (sflags & TS_TRI_A) inside = inside && ((lower != TA) ? k0 + slab_k <= i_base : k0 >= i_base + BM);
    if (sflags & TS_TRI_B) inside = inside && ((lower != TB) ? k0 >= j_base + BN : k0 + slab_k <= j_base);
    return inside;
}

// How a step with a triangular operand hands out its macro-tiles.  Their work depends on the
// row block (triangular A) or the column block (triangular B) only, so that index is made the
// slow one: consecutive workgroups, which the hardware deals round-robin to the shader engines
// of an XCD, are then equally long and every engine gets the same mix (with the row block as the
// fast index one engine got all the longest macro-tiles: 584 us for a launch of 16 diagonal
// steps instead of 300).  And where the work grows with the index (the triangle cuts the k range
// from above) the macro-tiles go out last to first, longest first.
struct MaskedOrder {
    bool reversed;        // hand out last to first
    bool rows_slow;       // row block = slow index (else the usual column-major order of macro-tiles)
};
template <bool TA, bool TB>
__device__ __forceinline__ MaskedOrder masked_order(const TileStep& st) {
    for (int q = 0; q < st.nseg; ++q) {
        const uint32_t f = st.seg[q].flags;
        const bool lower = f & TS_TRI_LOWER;
        if (f & TS_TRI_A) return MaskedOrder{lower != TA, true};
        if (f & TS_TRI_B) return MaskedOrder{lower == TB, false};
    }
    return MaskedOrder{false, false};
}

// The inner dimension of a pair as the fast kernel walks it: whole slab pairs.  Only a step of zero-padded
// tiles (TS_PADDED) has a k that this rounds up; the products with the padding are zero.
template <typename T>
__device__ __forceinline__ int whole_slab_pairs(int k) {
    constexpr int Q = 2 * FastShape<T>::SLAB_K;
    return (k + Q - 1) / Q * Q;
}

// MASK: the pack holds steps with triangular operands (separate kernel instantiation, so that
// the plain one carries no trace of the masking code).
template <typename T, bool TA, bool TB, bool MASK>
__device__ __forceinline__ void macro_tile_fast(const TileStep& st, int i_base, int j_base) {
    typedef typename Mfma<T>::acc_t acc_t;
    typedef FastShape<T> S;
    // two stages, one array per stage and operand so that the compiler can tell a copy into one
    // stage from the fragment reads of the other
    __shared__ __attribute__((aligned(1024))) T sA0[S::STAGE], sB0[S::STAGE], sA1[S::STAGE], sB1[S::STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS windows in SGPRs
    const int g = lane >> 4, r16 = lane & 15;
    const int wm = wave & 1, wn = wave >> 1;
    const int lda = st.lda, ldb = st.ldb;
    const int nseg = st.nseg;

    acc_t acc[4][S::NBJ];
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < S::NBJ; ++bj) acc[bi][bj] = acc_t{0, 0, 0, 0};
    const CopyLane<T, TA> copy_a(lda, i_base, wave, lane);
    const CopyLane<T, !TB> copy_b(ldb, j_base, wave, lane);

    // bytes from one slab of a tile to the next
    const uint32_t step_a = (uint32_t)((TA ? S::SLAB_K : S::SLAB_K * lda) * (int)sizeof(T));
    const uint32_t step_b = (uint32_t)((!TB ? S::SLAB_K : S::SLAB_K * ldb) * (int)sizeof(T));

    // Copy cursor: slab `pslab` of the k range [pkb, pke) of pair `pseg` is the next one to fetch; it starts
    // pa, pb bytes into the pair's tiles ta, tb (all of this is the same for every lane).
    int pseg = -1, pslab = 0, pkb = 0, pke = 0;
    __amdgpu_buffer_rsrc_t ta = tile_rsrc(st.seg[0].A), tb = tile_rsrc(st.seg[0].B);
    uint32_t pa = 0, pb = 0;
    // first slab of the next pair that has any (a masked pair may have none for this macro-tile)
    auto next_pair = [&]() -> bool {
        if constexpr (MASK) {
            for (++pseg; pseg < nseg; ++pseg) {
                masked_k_range<TA, TB>(st.seg[pseg].flags, whole_slab_pairs<T>(st.seg[pseg].k), i_base, j_base, pkb, pke);
                if (pke > pkb) break;
            }
            if (pseg >= nseg) return false;
            pa = (uint32_t)(pkb / S::SLAB_K) * step_a;
            pb = (uint32_t)(pkb / S::SLAB_K) * step_b;
        } else {
            if (++pseg >= nseg) return false;
            pke = whole_slab_pairs<T>(st.seg[pseg].k);
            pa = pb = 0;
        }
        ta = tile_rsrc(st.seg[pseg].A);
        tb = tile_rsrc(st.seg[pseg].B);
        pslab = 0;
        return true;
    };
    // `pend`: the cursor is on a slab (whose copies are still to be issued); false once the chain is exhausted.
    // advance() moves it to the next slab of the chain.  Only the step into another pair, once in a whole tile's
    // worth of slabs, takes a branch; the common case is three scalar additions and a compare.
    bool pend = false;
    auto advance = [&]() {
        ++pslab;
        pa += step_a;
        pb += step_b;
        if (__builtin_expect((MASK ? pkb : 0) + pslab * S::SLAB_K >= pke, 0)) pend = next_pair();
    };
    int total = 0;
    for (int q = 0; q < nseg; ++q) {
        int kb = 0, ke = whole_slab_pairs<T>(st.seg[q].k);
        if (MASK) masked_k_range<TA, TB>(st.seg[q].flags, whole_slab_pairs<T>(st.seg[q].k), i_base, j_base, kb, ke);
        total += (ke - kb) / S::SLAB_K;
    }
    pend = next_pair();
    if (pend) {
        dma_slab<T, TA>(ta, pa, lda, copy_a, sA0, wave);
        dma_slab<T, !TB>(tb, pb, ldb, copy_b, sB0, wave);
    }
    // Compute cursor: where in its pair the slab being multiplied lies and whether it needs masking (only
    // the masks need to know); `cur` describes the slab whose units are being issued, `nxt` the one after.
    struct SlabInfo { int k0; uint32_t mflags; };
    int cseg = pseg, cslab = 0, ckb = pkb, cke = pke;
    auto slab_info = [&]() -> SlabInfo {            // of the slab the compute cursor is on; moves the cursor on
        if constexpr (!MASK) return SlabInfo{0, 0u};
        const uint32_t cflags = cseg < nseg ? st.seg[cseg].flags : 0u;
        const int k0 = ckb + cslab * S::SLAB_K;
        const SlabInfo info{k0, slab_inside_triangle<TA, TB>(cflags, k0, S::SLAB_K, i_base, j_base) ? 0u : cflags};
        ++cslab;
        if (ckb + cslab * S::SLAB_K >= cke) {
            for (++cseg; cseg < nseg; ++cseg) {
                ckb = 0;
                cke = whole_slab_pairs<T>(st.seg[cseg].k);
                masked_k_range<TA, TB>(st.seg[cseg].flags, whole_slab_pairs<T>(st.seg[cseg].k), i_base, j_base, ckb, cke);
                if (cke > ckb) break;
            }
            cslab = 0;
        }
        return info;
    };
    FastRegs<T> R;
    constexpr int NU = FastRegs<T>::NU;
    const LaneBase<T, TA> lane_a(wm * 64, g, r16);
    const LaneBase<T, !TB> lane_b(wn * S::WAVE_N, g, r16);
    // One slab: units 0 .. NU - 2 each request the values of the unit after them and multiply their own; then,
    // with the values of the last unit in registers, nothing of this stage is needed any more: the wave waits
    // for its own copies into the other stage, meets the other waves at the barrier (after which that stage is
    // complete and this one is free), moves the copy cursor on to the slab after next, requests the first values
    // of the next slab -- and only then issues the MFMAs of its last unit, which cover all of that.
    // The copies of the slab the cursor is on go into the stage that is not being read: the first ones right
    // after the barrier (into the stage just freed), the rest, if the shape says so, with the first units of the
    // next slab (see FastShape::COPY_PP).
    // `more`: another slab follows.
    constexpr int LAST_POS = (S::DMA_PER_WAVE - 1) / S::COPY_PP - 1;
    static_assert(LAST_POS < NU / 2, "the copies must be out by the middle of the slab");
    auto copies_at = [&](int pos, T* wa, T* wb) {
#pragma unroll
        for (int i = 0; i < S::DMA_PER_WAVE; ++i)
            if (i / S::COPY_PP - 1 == pos) {
                dma_piece<T, TA>(ta, pa, lda, copy_a, wa, wave, i);
                dma_piece<T, !TB>(tb, pb, ldb, copy_b, wb, wave, i);
            }
    };
    auto slab = [&](T* sa, T* sb, T* na, T* nb, SlabInfo cur, SlabInfo nxt, bool more) {
#pragma unroll
        for (int u = 0; u + 1 < NU; ++u) {
            lds_fence();
            unit_load<T, TA, TB>(R, sa, sb, u + 1, lane_a, lane_b);
            if (u <= LAST_POS && pend) copies_at(u, na, nb);
            __builtin_amdgcn_sched_barrier(0);
            unit_mfma<T, TA, TB, MASK>(acc, R, u, wm, wn, g, r16, cur.mflags, cur.k0, i_base, j_base);
            if (sizeof(T) == 8 && (TA || !TB) && (u & 1)) {
                __builtin_amdgcn_sched_barrier(0);
                unit_load_late<T, TA, TB>(R, sa, sb, (u + 1) / 2, lane_a, lane_b);
            }
        }
        lds_fence();
        if (more) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's copies into the other stage have landed
            __syncthreads();
            advance();
            if (pend) copies_at(-1, sa, sb);
            unit_load<T, TA, TB>(R, na, nb, 0, lane_a, lane_b);
            __builtin_amdgcn_sched_barrier(0);
        }
        unit_mfma<T, TA, TB, MASK>(acc, R, NU - 1, wm, wn, g, r16, cur.mflags, cur.k0, i_base, j_base);
        if (sizeof(T) == 8 && (TA || !TB) && more) {
            __builtin_amdgcn_sched_barrier(0);
            unit_load_late<T, TA, TB>(R, na, nb, 0, lane_a, lane_b);
        }
    };
    // Slabs are processed in pairs (stage 0, then stage 1) with no exit in between, so that the
    // accumulators stay in one set of registers (the host only sends chains with an even count:
    // every k is a multiple of two slabs).
    if (total > 0) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();                          // stage 0 holds the first slab
        advance();
        if (pend) copies_at(-1, sA1, sB1);
        unit_load<T, TA, TB>(R, sA0, sB0, 0, lane_a, lane_b);
        unit_load_late<T, TA, TB>(R, sA0, sB0, 0, lane_a, lane_b);
        SlabInfo cur = slab_info();
        for (int pair = 0; pair < total / 2; ++pair) {
            SlabInfo nxt = slab_info();
            slab(sA0, sB0, sA1, sB1, cur, nxt, true);
            cur = nxt;
            const bool more = pair + 1 < total / 2;
            if (more) nxt = slab_info();
            slab(sA1, sB1, sA0, sB0, cur, nxt, more);
            cur = nxt;
        }
    }

    T* __restrict__ C = static_cast<T*>(st.C);
    const T* __restrict__ D = static_cast<const T*>(st.D);
    const T alpha = (T)st.alpha, beta = (T)st.beta;
    const bool use_c = (st.beta != 0.0);
    const int ldc = st.ldc;
    // Output-triangle mask (diagonal tiles of SYRK): +1 keeps i >= j, -1 keeps i <= j, 0 keeps all.
    const int tri = (st.flags & TS_C_LOWER) ? 1 : ((st.flags & TS_C_UPPER) ? -1 : 0);
    // C is m x n; a step of zero-padded tiles computes whole macro-tiles and stores what lies inside
    const int m_end = st.m, n_end = st.n;
    // Written in batches of RB accumulator rows of one 16-column block (RB x 4 values per lane of C, of the addend
    // D and of the result).  The loads of the next batch are issued before the stores of this one, so that the
    // epilogue pays one memory latency and not one per batch (every workgroup of a launch gets here at about the same
    // time: the loads of a batch then take a microsecond or two to come back); and a macro-tile that lies wholly
    // inside C and has no triangle to respect runs without the per-element tests (PRED = false).  Worth 0.6 % of
    // an fp32 launch of 8 k-tiles (more of shorter ones); nothing measurable in fp64, whose batches are half as deep.
    constexpr int RB = sizeof(T) == 8 ? 1 : 2;
    constexpr int NB = S::NBJ * 4 / RB;
    auto epilogue = [&](auto pred_tag) {
        constexpr bool PRED = decltype(pred_tag)::value;
        T cv[2][RB][4], dv[2][RB][4];
        auto row_of = [&](int bi) { return i_base + wm * 64 + bi * 16 + r16; };
        auto col_of = [&](int b, int r) { return j_base + wn * S::WAVE_N + (b / (4 / RB)) * 16 + Mfma<T>::drow((b % (4 / RB)) * RB + r, g); };
        auto keep = [&](int i, int j) { return !PRED || (tri * (i - j) >= 0 && i < m_end && j < n_end); };
        auto load = [&](int b, int buf) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi) {
                    const int i = row_of(bi), j = col_of(b, r);
                    const bool k = keep(i, j);
                    cv[buf][r][bi] = (use_c && k) ? C[(size_t)i + (size_t)j * ldc] : T(0);
                    dv[buf][r][bi] = (D && k) ? D[(size_t)i + (size_t)j * ldc] : T(0);
                }
        };
        load(0, 0);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b + 1 < NB) load(b + 1, (b + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi) {
                    const int i = row_of(bi), j = col_of(b, r);
                    T v = alpha * acc[bi][b / (4 / RB)][(b % (4 / RB)) * RB + r] + dv[b & 1][r][bi];
                    if (use_c) v += beta * cv[b & 1][r][bi];
                    if (keep(i, j)) C[(size_t)i + (size_t)j * ldc] = v;
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (tri == 0 && i_base + BM <= m_end && j_base + BN <= n_end) epilogue(std::false_type{});
    else epilogue(std::true_type{});
}

// MODE 0: fast path (the host has checked with step_is_fast() that every step of the pack is made
//         of whole macro-tiles with aligned operands and whole slab pairs in k), no operand masks;
// MODE 1: fast path with triangular operand masks;
// MODE 2: general path, everything else with predication.
enum { MODE_FAST = 0, MODE_FAST_MASKED = 1, MODE_GENERAL = 2 };

template <typename T, int MODE>
constexpr int kernel_threads() { return MODE == MODE_GENERAL ? NTHREADS : FastShape<T>::THREADS; }
// waves per SIMD the register budget is cut for: two workgroups per CU in every case
template <typename T, int MODE>
constexpr int kernel_waves_per_simd() { return MODE == MODE_GENERAL ? 2 : 2 * FastShape<T>::WAVES / 4; }

template <typename T, bool TA, bool TB, int MODE>
__global__ __launch_bounds__((kernel_threads<T, MODE>()), (kernel_waves_per_simd<T, MODE>()))
void tile_steps_kernel(const LaunchPack pack) {
    // XCD-aware virtual workgroup index: XCD x gets the contiguous range [x*per, (x+1)*per).
    const uint32_t per = gridDim.x / NXCD;
    const uint32_t v = (blockIdx.x % NXCD) * per + blockIdx.x / NXCD;
    if (v >= pack.total_wg) return;

    int s = 0;
    while (s + 1 < pack.nsteps && pack.step[s + 1].wg_begin <= v) ++s;
    const TileStep& st = pack.step[s];

    uint32_t local = v - st.wg_begin;
    const uint32_t tiles_m = (uint32_t)(st.m + BM - 1) / BM;
    int i_base = (int)(local % tiles_m) * BM;
    int j_base = (int)(local / tiles_m) * BN;
    if (MODE == MODE_FAST_MASKED) {
        const uint32_t tiles_n = (uint32_t)(st.n + BN - 1) / BN;
        const MaskedOrder order = masked_order<TA, TB>(st);
        if (order.reversed) local = tiles_m * tiles_n - 1 - local;
        i_base = (int)(order.rows_slow ? local / tiles_n : local % tiles_m) * BM;
        j_base = (int)(order.rows_slow ? local % tiles_n : local / tiles_m) * BN;
    }
    // Diagonal tile of SYRK / SYR2K (Eq. 1b): only the macro-tiles that touch the triangle of C that the step reads and
    // writes have workgroups (36 of the 64 of a 1024 x 1024 tile), numbered column by column as macro_tiles() counts them.
    if (st.flags & (TS_C_LOWER | TS_C_UPPER)) {
        const uint32_t tiles_n = (uint32_t)(st.n + BN - 1) / BN;
        uint32_t rest = v - st.wg_begin, i = 0, j = 0;
        for (; j < tiles_n; ++j) {
            const uint32_t count = (st.flags & TS_C_LOWER) ? (tiles_m > j ? tiles_m - j : 0) : (j + 1 < tiles_m ? j + 1 : tiles_m);
            if (rest < count) {
                i = (st.flags & TS_C_LOWER) ? j + rest : rest;
                break;
            }
            rest -= count;
        }
        i_base = (int)i * BM;
        j_base = (int)j * BN;
    }
    if (MODE == MODE_GENERAL)
        macro_tile<T, TA, TB>(st, i_base, j_base);
    else
        macro_tile_fast<T, TA, TB, MODE == MODE_FAST_MASKED>(st, i_base, j_base);
}

// Host-side launcher.  dtype: 0 = fp64, 1 = fp32; mode: see above.  The pack's wg_begin / total_wg
// must be filled, and mode must be MODE_GENERAL unless step_is_fast() holds for every step.
hipError_t launch_tile_steps(int dtype, bool ta, bool tb, int mode, const LaunchPack& pack, hipStream_t stream) {
    if (pack.nsteps <= 0 || pack.total_wg == 0) return hipSuccess;
    const uint32_t grid = NXCD * ((pack.total_wg + NXCD - 1) / NXCD);
#define BLASX_LAUNCH_MODE(T, TA, TB, MODE) \
    hipLaunchKernelGGL((tile_steps_kernel<T, TA, TB, MODE>), dim3(grid), dim3(kernel_threads<T, MODE>()), 0, stream, pack)
#define BLASX_LAUNCH(T, TA, TB)                                             \
    do {                                                                    \
        if (mode == MODE_FAST) BLASX_LAUNCH_MODE(T, TA, TB, MODE_FAST);     \
        else if (mode == MODE_FAST_MASKED) BLASX_LAUNCH_MODE(T, TA, TB, MODE_FAST_MASKED); \
        else BLASX_LAUNCH_MODE(T, TA, TB, MODE_GENERAL);                    \
    } while (0)
    if (dtype == 0) {
        if (!ta && !tb) BLASX_LAUNCH(double, false, false);
        else if (!ta && tb) BLASX_LAUNCH(double, false, true);
        else if (ta && !tb) BLASX_LAUNCH(double, true, false);
        else BLASX_LAUNCH(double, true, true);
    } else {
        if (!ta && !tb) BLASX_LAUNCH(float, false, false);
        else if (!ta && tb) BLASX_LAUNCH(float, false, true);
        else if (ta && !tb) BLASX_LAUNCH(float, true, false);
        else BLASX_LAUNCH(float, true, true);
    }
    return hipGetLastError();
}

// Every instantiation for one element type with an empty pack: each workgroup finds its virtual index
// beyond total_wg = 0 and returns at once.  Makes the runtime load the kernels ahead of their first use.
hipError_t launch_tile_steps_empty(int dtype, hipStream_t stream) {
    LaunchPack pack = {};             // nsteps = 0, total_wg = 0
    const uint32_t grid = NXCD;
    for (int mode = MODE_FAST; mode <= MODE_GENERAL; ++mode) {
        for (int v = 0; v < 4; ++v) {
            const bool ta = v & 1, tb = v & 2;
            if (dtype == 0) {
                if (!ta && !tb) BLASX_LAUNCH(double, false, false);
                else if (!ta && tb) BLASX_LAUNCH(double, false, true);
                else if (ta && !tb) BLASX_LAUNCH(double, true, false);
                else BLASX_LAUNCH(double, true, true);
            } else {
                if (!ta && !tb) BLASX_LAUNCH(float, false, false);
                else if (!ta && tb) BLASX_LAUNCH(float, false, true);
                else if (ta && !tb) BLASX_LAUNCH(float, true, false);
                else BLASX_LAUNCH(float, true, true);
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}
#undef BLASX_LAUNCH
#undef BLASX_LAUNCH_MODE

}  // namespace blasx
