/*
 * blasx.h -- C ABI of the single-GPU tile level-3 BLAS for MI355X (gfx950).
 *
 * The routines compute on HOST-resident matrices: the output is cut into T x T tile tasks
 * (paper Section IV.A), operand tiles stream over the host link into a tile cache in HBM
 * (Section IV.B, Alg. 2), every tile step runs as a hand-written MFMA kernel, and finished
 * tiles are written back to the host matrix (Section IV.D).  A call returns after the last
 * tile has landed in host memory, as a CPU BLAS would (Section I: legacy-BLAS compatible).
 *
 * Conventions
 *   - All matrix pointers are HOST pointers owned by the caller.  They may be pageable, but
 *     only page-locked memory (blasx_host_alloc, hipHostMalloc, torch pin_memory) gives
 *     asynchronous DMA; the paper likewise page-locks its matrices (Section V.A).
 *   - Enum values are those of the C BLAS interface:
 *       Order 101 row-major / 102 column-major;  Trans 111 none / 112 transpose / 113 conjugate
 *       transpose (= transpose for real data);  Uplo 121 upper / 122 lower;
 *       Diag 131 non-unit / 132 unit;  Side 141 left / 142 right.
 *   - Leading dimensions are in elements.  Dimensions are int; all offsets are computed in
 *     size_t, so matrices beyond 2^31 elements are fine.
 *   - Input matrices are only read.  Outputs must not overlap inputs.
 *   - Return value: 0 on success; -k if the k-th argument is invalid (1-based, as counted in
 *     the prototype); a positive BLASX_ERR_* code for run-time failures.  Nothing is written
 *     to the output when an argument error is returned.
 *   - The library is not re-entrant: one call at a time per process.
 */
#ifndef BLASX_H
#define BLASX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    BLASX_ROW_MAJOR = 101, BLASX_COL_MAJOR = 102,
    BLASX_NO_TRANS = 111, BLASX_TRANS = 112, BLASX_CONJ_TRANS = 113,
    BLASX_UPPER = 121, BLASX_LOWER = 122,
    BLASX_NON_UNIT = 131, BLASX_UNIT = 132,
    BLASX_LEFT = 141, BLASX_RIGHT = 142
};

enum {
    BLASX_OK = 0,
    BLASX_ERR_NOT_INITIALIZED = 1,  /* blasx_init has not been called (or shutdown was) */
    BLASX_ERR_ARENA_TOO_SMALL = 2,  /* the tile cache cannot hold the minimum working set */
    BLASX_ERR_DEVICE = 3,           /* a HIP call failed; see blasx_last_error() */
    BLASX_ERR_CONFIG = 4,           /* invalid tile size / stream count / option value */
    BLASX_ERR_NO_MEMORY = 5,        /* host allocation failed */
    BLASX_ERR_UNSUPPORTED = 6,      /* valid BLAS arguments that this build does not cover */
    BLASX_ERR_TOO_LARGE = 7         /* blasx_dgemm_noalloc: the operands do not fit the static scratch */
};

/* ------------------------------------------------------------------ level-3 routines -- */

/* C <- alpha * op(A) * op(B) + beta * C                (paper Eq. 1a, task per C tile)
 * op(A) is M x K, op(B) is K x N, C is M x N.  beta == 0: C is not read.
 * alpha == 0: A and B are not read.  Arguments 1..14 in prototype order. */
int blasx_dgemm(int Order, int TransA, int TransB, int M, int N, int K, double alpha,
                const double* A, int lda, const double* B, int ldb, double beta, double* C, int ldc);
int blasx_sgemm(int Order, int TransA, int TransB, int M, int N, int K, float alpha,
                const float* A, int lda, const float* B, int ldb, float beta, float* C, int ldc);

/* blasx_dgemm for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, same error codes as
 * blasx_dgemm, but the tile slots live in an array that is part of the library's device image
 * (256 MiB per GPU the library runs on, held until the process ends) instead of the arena given to
 * blasx_init, and the call makes no hipMalloc, hipFree, stream or event creation and no other allocating
 * call: blasx_init (which must have been called, on this device) has looked the array's address up
 * and created the events it uses.
 *   - A, B and C must be page-locked (BLASX_ERR_UNSUPPORTED otherwise: the runtime would stage
 *     pageable memory through buffers of its own).
 *   - Tile edge: the configured one (blasx_set_tile) if it is between 16 and 512, else 512.  Every tile of
 *     A, B and C gets a slot of its own and nothing is evicted, so the call is accepted when
 *         nt(M) nt(K) + nt(K) nt(N) + nt(M) nt(N) + 8 <= 256 MiB / (T * T * 8 bytes),   nt(x) = ceil(x / T)
 *     (T = 512: 128 slots, e.g. M = N = K <= 3072 rounded down to what the count allows: 2560), and
 *     refused with BLASX_ERR_TOO_LARGE (text in blasx_last_error) otherwise.  Nothing is computed then.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents; nothing in
 *     it needs to start at zero (an accumulator tile is written before it is read).  Calls that
 *     overlap on one GPU would race: like the rest of the library, one call at a time.
 *   - "persist", "profile" and blasx_set_cache_bytes do not apply; the other options do. */
int blasx_dgemm_noalloc(int Order, int TransA, int TransB, int M, int N, int K, double alpha,
                        const double* A, int lda, const double* B, int ldb, double beta, double* C, int ldc);

/* C <- alpha * A * A^T + beta * C (Trans = none, A is N x K) or
 * C <- alpha * A^T * A + beta * C (Trans = transpose, A is K x N)      (paper Eq. 1b)
 * Only the Uplo triangle of C (with its diagonal) is read or written; the other triangle of
 * the host matrix is left bit-identical. */
int blasx_dsyrk(int Order, int Uplo, int Trans, int N, int K, double alpha,
                const double* A, int lda, double beta, double* C, int ldc);
int blasx_ssyrk(int Order, int Uplo, int Trans, int N, int K, float alpha,
                const float* A, int lda, float beta, float* C, int ldc);

/* C <- alpha * (A * B^T + B * A^T) + beta * C (Trans = none, A and B are N x K) or
 * C <- alpha * (A^T * B + B^T * A) + beta * C (Trans = transpose, A and B are K x N)   (paper Eq. 1e)
 * Only the Uplo triangle of C (with its diagonal) is read or written; the other triangle of
 * the host matrix is left bit-identical.  Arguments 1..13 in prototype order. */
int blasx_dsyr2k(int Order, int Uplo, int Trans, int N, int K, double alpha,
                 const double* A, int lda, const double* B, int ldb, double beta, double* C, int ldc);
int blasx_ssyr2k(int Order, int Uplo, int Trans, int N, int K, float alpha,
                 const float* A, int lda, const float* B, int ldb, float beta, float* C, int ldc);

/* C <- alpha * A * B + beta * C (Side = left, A is M x M) or
 * C <- alpha * B * A + beta * C (Side = right, A is N x N), A symmetric, B and C M x N  (paper Eq. 1f)
 * Only the Uplo triangle of A (with its diagonal) is read; the other triangle may hold anything.
 * Tiles of A outside the stored triangle are made on the device from the stored ones (diagonal
 * tiles completed by reflection, the others transposed), in cache slots of their own. */
int blasx_dsymm(int Order, int Side, int Uplo, int M, int N, double alpha,
                const double* A, int lda, const double* B, int ldb, double beta, double* C, int ldc);
int blasx_ssymm(int Order, int Side, int Uplo, int M, int N, float alpha,
                const float* A, int lda, const float* B, int ldb, float beta, float* C, int ldc);

/* Solve op(A) * X = alpha * B (Side = left, A is M x M) or X * op(A) = alpha * B (right,
 * A is N x N); X overwrites B (M x N).                                  (paper Eq. 1c, with
 * alpha placed as in the BLAS standard).  Only the Uplo triangle of A is read; with
 * Diag = unit the diagonal is not read either. */
int blasx_dtrsm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha,
                const double* A, int lda, double* B, int ldb);
int blasx_strsm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, float alpha,
                const float* A, int lda, float* B, int ldb);

/* B <- alpha * op(A) * B (left) or alpha * B * op(A) (right)            (paper Eq. 1d, alpha on
 * every term).  Same triangle rules as blasx_dtrsm. */
int blasx_dtrmm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, double alpha,
                const double* A, int lda, double* B, int ldb);
int blasx_strmm(int Order, int Side, int Uplo, int TransA, int Diag, int M, int N, float alpha,
                const float* A, int lda, float* B, int ldb);

/* ------------------------------------------------------------------ run-time control -- */

/* Hand the library its device resources (paper Section IV.E: one pre-allocated chunk, no
 * per-tile device malloc).
 *   arena        DEVICE pointer to arena_bytes of HBM that stays valid until blasx_shutdown
 *                (e.g. a torch uint8 tensor).  NULL: the library allocates arena_bytes itself.
 *   hip_streams  HOST array of nstreams hipStream_t handles (e.g. torch streams), used in
 *                this order: compute, host-to-device, device-to-host, second host-to-device.
 *                NULL: the library creates nstreams streams.  All at default priority.
 *   nstreams     2..4, or 0 for the measured best (4; hip_streams must then be NULL or hold
 *                4 handles).  With 2, both copy directions share one stream; with 3 each direction
 *                has its own; with 4 inbound copies alternate between two streams.
 * Must be called with the target device current.  Calling it again re-initialises; an arena
 * that the library allocated itself is kept and used again when it is large enough (freeing
 * gigabytes of device memory halves the outbound copy rate until the driver has cleared them:
 * 1.5 s for 48 GiB), and is freed by blasx_shutdown. */
int blasx_init(void* arena, size_t arena_bytes, void* const* hip_streams, int nstreams);
int blasx_shutdown(void);

/* Tile edge T (paper Section V.B: the one tuning parameter).  Multiple of 16, 16..8192, or 0: chosen per
 * call from the extent of the output matrix, the element type and the room in the tile cache (1024 for
 * most double-precision calls, 1024 or 2048 in single precision, 512 or 2048 for some triangular
 * orders; halved until 64 tiles fit in the cache).  The choice of the latest call is
 * blasx_get_option("last_tile").  The default is 1024.  With T a multiple of 128 matrices of any order
 * run in the fast kernels (ragged edge tiles are kept zero-padded in the tile cache); with another T every
 * tile step takes the slower bounds-checked kernel (blasx_stats.steps_general counts them). */
int blasx_set_tile(int T);
/* Number of streams the scheduler uses (paper Section IV.D: tasks progress on concurrent
 * streams; its experiments use 4).  n = 2..4 with the roles listed at blasx_init, or 0 for the
 * measured best (4).  The streams handed to (or made by) blasx_init keep their roles: fewer
 * streams leave the later ones idle, more takes further streams of the library's own -- no
 * stream is created anew for a role that had one, because which hardware queue a new stream
 * lands on depends on what was created before it and two roles sharing a queue serialise.
 * BLASX_ERR_NOT_INITIALIZED before blasx_init; BLASX_ERR_CONFIG when n is out of range or
 * exceeds the number of caller-owned streams given to blasx_init.  Only between calls; the
 * tile cache (option "persist") is kept.  blasx_get_option("streams") reads it back. */
int blasx_set_streams(int n);
/* Cap on the bytes of the arena that the tile cache may use (0 = all of it); lowers the
 * number of tile slots so that eviction (Alg. 2, Dequeue) can be exercised. */
int blasx_set_cache_bytes(size_t cap);
/* Scheduling knobs.  name is one of
 *   "group"    tile tasks that run together and advance k-step by k-step; 0 (default): chosen per
 *              call from the number of tasks (2 .. 16; 16 for the triangular routines); the choice of
 *              the latest call is "last_group"
 *   "kchain"   consecutive k-steps of a task fused into one launch (1..8; 1 = the paper's one kernel
 *              per (i,j,k)); 0 (default): chosen per call (8 in the wide schedule when the k loop is
 *              long enough, else 4 .. 6; 1 .. 3 for the triangular product up to 16 x 16 tiles; the
 *              wide triangular solve always takes one k-step per round); "last_kchain"
 *   "wide"     least number of k-tiles per task from which ALL tasks of a call run together and
 *              advance k-chunk by k-chunk (an outer-product order: enough products per tile copied
 *              from the first launch on, C tiles fetched only for a task's last launch, results
 *              leaving during the whole last round), provided the cache has room for an accumulator
 *              tile per output tile; 0: never (tasks run to completion in groups, the paper's
 *              scheme).  Default 11; the triangular routines use it from a third of the value.
 *              "last_wide" tells whether the latest call ran that way
 *   "ramp"     wide schedule: k-steps per task in the first round (1..8; 8 = as in every other
 *              round).  0 (default): the steps left over when the k loop is cut into rounds come
 *              first rather than last, and when nothing is left over the first full round is split
 *              into 2 steps and the rest.  The choice of the latest call is "last_ramp"
 *   "prefetch" wide schedule: inbound copies are started this many launches ahead (default 24)
 *   "merge"    most whole tiles that one inbound copy may carry (1..8; 0, the default: as many as make
 *              32 MiB, between 2 and 8: 4 tiles of 1024 x 1024 doubles).  Tiles that lie side
 *              by side in a block row of a column-major host matrix and go to neighbouring slots of the
 *              tile cache are one strided copy: the copy engine pauses between copies, not inside one.
 *              1: one copy per tile (the paper's scheme)
 *   "late_c"   1 (default): a call in the grouped schedule whose tiles all fit the cache beside two slots per
 *              running task fetches the host tile of C for a task's last launch only (as the wide schedule
 *              always does) and cuts the k loop into launches of two k-tiles; 0: C comes in with the task's
 *              first launch (the paper's order), launches of four k-tiles
 *   "row_order" 1 (default): the same calls take their tasks block row by block row of C, whatever
 *              "sb_rows" / "sb_cols" / "shells" say; 0: always in the queue order those give
 *   "stagger_panels", "stagger_lag"  wide triangular solve and triangular product: the right-hand sides
 *              are cut into stagger_panels (default 2) independent panels of block columns (block rows
 *              for Side = Right), each running stagger_lag rounds (solve: one round = one block row of
 *              the triangle; product: one launch per task) behind the one before, so that the short last
 *              rounds of one panel, whose results leave in a burst, run under the product-rich first
 *              rounds of the next.  stagger_lag 0 (default): half of the rounds (product: one round
 *              when it has fewer than five) when the device rather than the link bounds the call, else
 *              none; -1: none
 *   "tail_cut" wide schedule: the last sixteen tasks of the last round are launched this many at a time
 *              (default 4; 0 or 16: sixteen, like every other launch), so that most of their result tiles
 *              leave while a kernel still runs
 *   "depth"    launches the host may run ahead of the device (>= 1)
 *   "rs"       reservation-station size: queued tasks whose priorities are compared (>= group)
 *   "priority" 1 (default): the next task to start is the one of the reservation station with the
 *              most operand tiles already cached (paper Eq. 2; ties go to queue order);
 *              0: queue order, for comparison
 *   "sb_rows", "sb_cols"  super-block shape used to order the task queue
 *   "shells"   1: super-blocks are visited in growing square shells, 0: block row by block row
 *   "profile"  1: time every launch with events (adds two event records per launch);
 *              2: also put an event before and after every tile copy and dissect each call as the
 *              paper's time profile does (Section V.A): t_kernel_busy_s, t_copy_unoverlapped_s
 *              and t_device_span_s of blasx_stats
 *   "persist"  1: the tile cache outlives the call (see below); 0 (default): it is dropped
 *              when a call returns
 * Returns BLASX_ERR_CONFIG for an unknown name or an out-of-range value. */
int blasx_set_option(const char* name, long value);
/* Reads a knob back; also "tile", "cached_tiles" (blocks now held by the persistent cache) and
 * the choices of the latest call: "last_tile", "last_group", "last_kchain", "last_wide" (1: the
 * wide schedule ran), "last_ramp".  -1 for an unknown name. */
long blasx_get_option(const char* name);

/* Persistent tile cache (the paper's applications multiply by the same matrices call after
 * call, Section V.C; the paper does not say what happens to cached tiles between calls).
 * With "persist" = 1 operand tiles, and tiles derived from them (inverted or completed
 * diagonal tiles), stay in HBM after a call returns and are hits for later calls that name the
 * same host tile (address, leading dimension, extent, element size), least recently used
 * ones making room as usual.  The contract:
 *   - the library forgets by itself every cached tile that shares an element with a matrix it
 *     writes (the output of any call, before and after the call; results of a triangular
 *     solve stay cached, they equal the host copy);
 *   - the caller must tell the library before the next call when it has changed, freed or
 *     re-used the memory of a matrix that was an operand of an earlier call, by one of:
 *       blasx_invalidate(ptr, bytes)       every cached tile touching [ptr, ptr + bytes)
 *       blasx_invalidate_matrix(A, ld, rows, cols, elem_size)
 *                                          every cached tile sharing an element with the
 *                                          rows x cols column-major matrix at A (for a
 *                                          row-major matrix pass its columns as rows); exact
 *                                          for views of one parent matrix with the same ld
 *       blasx_invalidate_all()             everything
 *     A stale tile is not detected: results are then computed from the old values.
 *   - changing the tile size, the cache cap or the element size of the calls empties the
 *     cache; blasx_init / blasx_shutdown / "persist" = 0 drop it.
 * The three calls return 0, or -k for a bad k-th argument; they are cheap no-ops when nothing
 * is cached.  Not thread-safe, like the rest of the library. */
int blasx_invalidate(const void* ptr, size_t bytes);
int blasx_invalidate_matrix(const void* A, int ld, int rows, int cols, int elem_size);
int blasx_invalidate_all(void);

/* Page-locked host memory for matrices (hipHostMalloc).  Returns NULL on failure. */
void* blasx_host_alloc(size_t bytes);
int   blasx_host_free(void* p);

typedef struct blasx_stats {
    uint64_t calls;          /* level-3 calls since the last reset */
    uint64_t tasks;          /* C tiles solved */
    uint64_t tile_steps;     /* (i, j, k) steps executed */
    uint64_t launches;       /* kernel launches */
    uint64_t hits;           /* tile-cache hits (operand tiles) */
    uint64_t misses;         /* tile-cache misses (each one is an inbound tile copy) */
    uint64_t evictions;      /* blocks discarded to make room */
    uint64_t refetches;      /* misses on a tile that had been evicted before */
    uint64_t copies_h2d, copies_d2h;
    uint64_t bytes_h2d, bytes_d2h;
    uint64_t slot_waits;     /* times the host had to wait for a slot to become free */
    uint64_t peak_slots;     /* most tile slots in use at once */
    uint64_t profiled_launches;
    double   flops;          /* floating-point operations of the executed tile steps */
    double   t_total_s;      /* wall time inside level-3 calls */
    double   t_issue_s;      /* of which: host scheduling/issue time (t_total_s - t_wait_s) */
    double   t_kernel_s;     /* sum of event-timed launch durations ("profile" >= 1) */
    uint64_t invalidations;  /* cached tiles forgotten because their host copy changed (persistent cache) */
    double   t_wait_s;       /* of t_total_s: host blocked on the device (run-ahead bound reached, no free slot,
                                final drain) */
    /* The paper's time profile (Section V.A: computation / communication that is not overlapped /
     * other), from events on the device's own clock; filled with "profile" = 2 only: */
    double   t_kernel_busy_s;        /* time during which at least one tile kernel ran (COMPT) */
    double   t_copy_unoverlapped_s;  /* time during which a tile copy ran, in either direction, and no
                                        kernel did (COMM) */
    double   t_device_span_s;        /* first device operation of each call to its last; the rest of it
                                        is OTHER = span - COMPT - COMM */
    uint64_t steps_general;  /* of tile_steps: run by the bounds-checked general kernel instead of a fast one
                                (only with a tile edge that is not a multiple of 128) */
    uint64_t transfers_h2d;  /* inbound copies handed to the copy engine; copies_h2d counts the tiles they carried */
} blasx_stats;

int blasx_get_stats(blasx_stats* out);
int blasx_reset_stats(void);

const char* blasx_strerror(int rc);
/* Text of the most recent device error ("" if none). */
const char* blasx_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BLASX_H */
