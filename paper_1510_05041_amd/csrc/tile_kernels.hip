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
// Shape: 512 threads = 8 waves (2 x 4) per workgroup, each wave owning 64 x 32 of the macro-tile
// (4 x 2 MFMA blocks), two workgroups per CU = 4 waves per SIMD to cover barrier and LDS latencies.
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

constexpr int FAST_THREADS = 512;
constexpr int FAST_WAVES = 8;
constexpr int DMA_PER_WAVE = 16 / FAST_WAVES;   // wave-wide copies per operand slab and wave

template <typename T> struct FastShape {
    static constexpr int EPC = 16 / (int)sizeof(T);      // elements per 16-byte chunk
    static constexpr int SLAB_K = 8 * EPC;               // k depth of one slab
    static constexpr int ROWS_PER_COPY = 1024 / (128 * (int)sizeof(T));   // k rows one wave-wide copy covers
    static constexpr int LANES_PER_ROW = 64 / ROWS_PER_COPY;
    static constexpr int STAGE = 128 * SLAB_K;           // elements per operand stage (16 KB)
};

template <typename T, bool KCONTIG>
__device__ __forceinline__ const T* dma_origin(const T* p, int ld, int mn_base, int wave, int lane) {
    typedef FastShape<T> S;
    if (!KCONTIG) {
        const int row = wave * DMA_PER_WAVE * S::ROWS_PER_COPY + lane / S::LANES_PER_ROW;
        // fp32: a 4-byte fragment read serves 32 lanes per pass = two lane groups g, whose rows are
        // 4 apart and would start at the same bank; every other group of 4 rows is therefore stored
        // with its columns shifted by half the banks (col ^ 16).  All rows of one wave's copies
        // fall in the same group of 4, so the shift is the same for the whole wave.
        const int chunk = (lane % S::LANES_PER_ROW) ^ (sizeof(T) == 4 ? 4 * ((row >> 2) & 1) : 0);
        return p + (size_t)(mn_base + chunk * S::EPC) + (size_t)row * ld;
    }
    const int m = lane >> 3, q = (lane & 7) ^ m;
    return p + (size_t)(S::EPC * q) + (size_t)(mn_base + wave * DMA_PER_WAVE * 8 + m) * ld;
}

// This wave's copies of one operand slab into the operand's 16 KB LDS window `stage`.
template <typename T, bool KCONTIG>
__device__ __forceinline__ void dma_slab(const T* origin, int ld, T* stage, int wave) {
    typedef FastShape<T> S;
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
        const T* src = origin + (size_t)(KCONTIG ? 8 * i : S::ROWS_PER_COPY * i) * ld;
        T* dst = stage + (wave * DMA_PER_WAVE + i) * (1024 / (int)sizeof(T));
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)dst, 16, 0, 0);
    }
}

// Fragments of MFMA group (c, h): one element per 16 x 16 block.
template <typename T, bool KCONTIG, int NB>
__device__ __forceinline__ void frag_read(T (&f)[NB], const T* stage, int c, int h, int base, int g, int r16) {
    typedef FastShape<T> S;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (!KCONTIG) {
            const int swz = sizeof(T) == 4 ? 16 * (g & 1) : 0;      // see dma_origin
            f[b] = stage[(4 * S::EPC * c + S::EPC * g + h) * 128 + ((base + b * 16 + r16) ^ swz)];
        } else {
            const int mn = base + b * 16 + r16;
            f[b] = stage[(mn * 8 + ((4 * c + g) ^ (r16 & 7))) * S::EPC + h];
        }
    }
}

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

// MFMAs of one slab.  MASK: one operand of this chained pair is a diagonal tile of a triangular
// matrix (sflags says which and how); its fragments are masked on their way out of LDS, so what
// the other triangle holds in memory never reaches an MFMA.  k0 = k offset of the slab in the pair.
template <typename T, bool TA, bool TB, bool MASK>
__device__ __forceinline__ void compute_stage(typename Mfma<T>::acc_t (&acc)[4][2], const T* sa, const T* sb,
                                              int wm, int wn, int g, int r16, uint32_t sflags, int k0,
                                              int i_base, int j_base) {
    typedef FastShape<T> S;
    constexpr int NGROUP = 2 * S::EPC;
    auto load_group = [&](T (&fa)[4], T (&fb)[2], int t) {
        const int c = t / S::EPC, h = t % S::EPC;
        frag_read<T, TA, 4>(fa, sa, c, h, wm * 64, g, r16);
        frag_read<T, !TB, 2>(fb, sb, c, h, wn * 32, g, r16);
        if (MASK) {
            const int kg = k0 + 4 * S::EPC * c + S::EPC * g + h;
            if (sflags & TS_TRI_A) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int i = i_base + wm * 64 + b * 16 + r16;
                    fa[b] = TA ? tri_select(fa[b], kg, i, sflags) : tri_select(fa[b], i, kg, sflags);
                }
            }
            if (sflags & TS_TRI_B) {
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int j = j_base + wn * 32 + b * 16 + r16;
                    fb[b] = TB ? tri_select(fb[b], j, kg, sflags) : tri_select(fb[b], kg, j, sflags);
                }
            }
        }
    };
    if constexpr (sizeof(T) == 4) {
        // fp32: the four MFMA groups h = 0..3 of one c share their 16-byte chunks, so a k-contiguous
        // operand is read one whole chunk per lane (conflict-free for 16-byte reads thanks to the
        // XOR in the layout; four separate 4-byte reads of it would collide four ways).  The unit
        // of the software pipeline is therefore (c, block row bi): 8 MFMAs (4 h x 2 bj) on the A
        // values of one block and the B values of c; the A values of the next unit are requested
        // before the MFMAs of this one, the B values of c = 1 during the first units of c = 0, so
        // that only three chunks per lane stand between the barrier and a wave's first MFMA.
        auto load_a = [&](T (&va)[4], int c, int bi) {
            if (TA) {
                const int mn = wm * 64 + bi * 16 + r16;
                const float4 v = reinterpret_cast<const float4*>(sa)[mn * 8 + ((4 * c + g) ^ (r16 & 7))];
                va[0] = v.x; va[1] = v.y; va[2] = v.z; va[3] = v.w;
            } else {
#pragma unroll
                for (int h = 0; h < 4; ++h) va[h] = sa[(16 * c + 4 * g + h) * 128 + ((wm * 64 + bi * 16 + r16) ^ (16 * (g & 1)))];
            }
            if (MASK && (sflags & TS_TRI_A)) {
                const int i = i_base + wm * 64 + bi * 16 + r16;
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const int kg = k0 + 16 * c + 4 * g + h;
                    va[h] = TA ? tri_select(va[h], kg, i, sflags) : tri_select(va[h], i, kg, sflags);
                }
            }
        };
        auto load_b = [&](T (&vb)[2][4], int c) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                if (!TB) {
                    const int mn = wn * 32 + b * 16 + r16;
                    const float4 v = reinterpret_cast<const float4*>(sb)[mn * 8 + ((4 * c + g) ^ (r16 & 7))];
                    vb[b][0] = v.x; vb[b][1] = v.y; vb[b][2] = v.z; vb[b][3] = v.w;
                } else {
#pragma unroll
                    for (int h = 0; h < 4; ++h) vb[b][h] = sb[(16 * c + 4 * g + h) * 128 + ((wn * 32 + b * 16 + r16) ^ (16 * (g & 1)))];
                }
                if (MASK && (sflags & TS_TRI_B)) {
                    const int j = j_base + wn * 32 + b * 16 + r16;
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const int kg = k0 + 16 * c + 4 * g + h;
                        vb[b][h] = TB ? tri_select(vb[b][h], j, kg, sflags) : tri_select(vb[b][h], kg, j, sflags);
                    }
                }
            }
        };
        T va[2][4], vb[2][2][4];
        load_b(vb[0], 0);
        load_a(va[0], 0, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = u >> 2, bi = u & 3, cur = u & 1;
            lds_fence();      // the values of this unit, requested one unit earlier, have arrived
            if (u + 1 < 8) load_a(va[cur ^ 1], (u + 1) >> 2, (u + 1) & 3);
            if (u == 1) load_b(vb[1], 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 4; ++h)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) acc[bi][bj] = Mfma<T>::run(vb[c][bj][h], va[cur][h], acc[bi][bj]);
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
    // fragments are double buffered: those of group t+1 are requested before the MFMAs of group t
    T fa[2][4], fb[2][2];
    load_group(fa[0], fb[0], 0);
#pragma unroll
    for (int t = 0; t < NGROUP; ++t) {
        const int cur = t & 1, nx = cur ^ 1;
        if (t + 1 < NGROUP) load_group(fa[nx], fb[nx], t + 1);
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj) acc[bi][bj] = Mfma<T>::run(fb[cur][bj], fa[cur][bi], acc[bi][bj]);
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

    acc_t acc[4][2];
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) acc[bi][bj] = acc_t{0, 0, 0, 0};

    const size_t step_a = TA ? (size_t)S::SLAB_K : (size_t)S::SLAB_K * lda;
    const size_t step_b = !TB ? (size_t)S::SLAB_K : (size_t)S::SLAB_K * ldb;

    // Copy cursor: slab `pslab` of the k range [pkb, pke) of pair `pseg` is the next one to fetch.
    int pseg = -1, pslab = 0, pkb = 0, pke = 0;
    const T* pa = nullptr;
    const T* pb = nullptr;
    // first slab of the next pair that has any (a masked pair may have none for this macro-tile)
    auto next_pair = [&]() -> bool {
        if constexpr (MASK) {
            for (++pseg; pseg < nseg; ++pseg) {
                masked_k_range<TA, TB>(st.seg[pseg].flags, st.seg[pseg].k, i_base, j_base, pkb, pke);
                if (pke > pkb) break;
            }
            if (pseg >= nseg) return false;
            pa = dma_origin<T, TA>(static_cast<const T*>(st.seg[pseg].A), lda, i_base, wave, lane) + (size_t)(pkb / S::SLAB_K) * step_a;
            pb = dma_origin<T, !TB>(static_cast<const T*>(st.seg[pseg].B), ldb, j_base, wave, lane) + (size_t)(pkb / S::SLAB_K) * step_b;
        } else {
            if (++pseg >= nseg) return false;
            pke = st.seg[pseg].k;
            pa = dma_origin<T, TA>(static_cast<const T*>(st.seg[pseg].A), lda, i_base, wave, lane);
            pb = dma_origin<T, !TB>(static_cast<const T*>(st.seg[pseg].B), ldb, j_base, wave, lane);
        }
        pslab = 0;
        return true;
    };
    // advance the copy cursor to the next slab of the chain; false when the chain is exhausted
    auto advance = [&]() -> bool {
        ++pslab;
        if ((MASK ? pkb : 0) + pslab * S::SLAB_K >= pke) return next_pair();
        pa += step_a;
        pb += step_b;
        return true;
    };
    int total = 0;
    for (int q = 0; q < nseg; ++q) {
        int kb = 0, ke = st.seg[q].k;
        if (MASK) masked_k_range<TA, TB>(st.seg[q].flags, st.seg[q].k, i_base, j_base, kb, ke);
        total += (ke - kb) / S::SLAB_K;
    }
    if (next_pair()) {
        dma_slab<T, TA>(pa, lda, sA0, wave);
        dma_slab<T, !TB>(pb, ldb, sB0, wave);
    }
    // Compute cursor: the slab now being multiplied (one behind the copy cursor); only the masks
    // need to know where in its pair a slab lies.
    int cseg = pseg, cslab = 0, ckb = pkb, cke = pke;
    uint32_t cflags = MASK && cseg < nseg ? st.seg[cseg].flags : 0;
    auto multiply = [&](const T* sa, const T* sb) {
        if constexpr (!MASK) {
            compute_stage<T, TA, TB, false>(acc, sa, sb, wm, wn, g, r16, 0u, 0, i_base, j_base);
            return;
        }
        const int k0 = ckb + cslab * S::SLAB_K;
        const uint32_t mflags = slab_inside_triangle<TA, TB>(cflags, k0, S::SLAB_K, i_base, j_base) ? 0u : cflags;
        compute_stage<T, TA, TB, MASK>(acc, sa, sb, wm, wn, g, r16, mflags, k0, i_base, j_base);
        if (MASK) {
            ++cslab;
            if (ckb + cslab * S::SLAB_K >= cke) {
                for (++cseg; cseg < nseg; ++cseg) {
                    ckb = 0;
                    cke = st.seg[cseg].k;
                    masked_k_range<TA, TB>(st.seg[cseg].flags, st.seg[cseg].k, i_base, j_base, ckb, cke);
                    if (cke > ckb) break;
                }
                cslab = 0;
                cflags = cseg < nseg ? st.seg[cseg].flags : 0;
            }
        }
    };
    // Slabs are processed in pairs (stage 0, then stage 1) with no exit in between, so that the
    // accumulators stay in one set of registers (the host only sends chains with an even count:
    // every k is a multiple of two slabs).
    for (int pair = 0; pair < total / 2; ++pair) {
        // stage 0 holds the current slab once every wave's copies have landed
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        advance();
        dma_slab<T, TA>(pa, lda, sA1, wave);
        dma_slab<T, !TB>(pb, ldb, sB1, wave);
        multiply(sA0, sB0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (advance()) {
            dma_slab<T, TA>(pa, lda, sA0, wave);
            dma_slab<T, !TB>(pb, ldb, sB0, wave);
        }
        multiply(sA1, sB1);
    }

    T* __restrict__ C = static_cast<T*>(st.C);
    const T* __restrict__ D = static_cast<const T*>(st.D);
    const T alpha = (T)st.alpha, beta = (T)st.beta;
    const bool use_c = (st.beta != 0.0);
    const int ldc = st.ldc;
    // Output-triangle mask (diagonal tiles of SYRK): +1 keeps i >= j, -1 keeps i <= j, 0 keeps all.
    const int tri = (st.flags & TS_C_LOWER) ? 1 : ((st.flags & TS_C_UPPER) ? -1 : 0);
#pragma unroll
    for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int rh = 0; rh < 4; rh += 2) {
            // half a 16-column block at a time: 8 values of C and 8 of the addend D in flight per lane
            T cv[2][4], dv[2][4];
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi) {
                    const int i = i_base + wm * 64 + bi * 16 + r16;
                    const int j = j_base + wn * 32 + bj * 16 + Mfma<T>::drow(rh + r, g);
                    const bool keep = tri * (i - j) >= 0;
                    cv[r][bi] = (use_c && keep) ? C[(size_t)i + (size_t)j * ldc] : T(0);
                    dv[r][bi] = (D && keep) ? D[(size_t)i + (size_t)j * ldc] : T(0);
                }
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi) {
                    const int i = i_base + wm * 64 + bi * 16 + r16;
                    const int j = j_base + wn * 32 + bj * 16 + Mfma<T>::drow(rh + r, g);
                    T v = alpha * acc[bi][bj][rh + r] + dv[r][bi];
                    if (use_c) v += beta * cv[r][bi];
                    if (tri * (i - j) >= 0) C[(size_t)i + (size_t)j * ldc] = v;
                }
            __builtin_amdgcn_sched_barrier(0);
        }
}

// MODE 0: fast path (the host has checked with step_is_fast() that every step of the pack is made
//         of whole macro-tiles with aligned operands and whole slab pairs in k), no operand masks;
// MODE 1: fast path with triangular operand masks;
// MODE 2: general path, everything else with predication.
enum { MODE_FAST = 0, MODE_FAST_MASKED = 1, MODE_GENERAL = 2 };

template <int MODE>
constexpr int kernel_threads() { return MODE == MODE_GENERAL ? NTHREADS : FAST_THREADS; }

template <typename T, bool TA, bool TB, int MODE>
__global__ __launch_bounds__((kernel_threads<MODE>()), (MODE == MODE_GENERAL ? 2 : 4))
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
    hipLaunchKernelGGL((tile_steps_kernel<T, TA, TB, MODE>), dim3(grid), dim3(kernel_threads<MODE>()), 0, stream, pack)
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
