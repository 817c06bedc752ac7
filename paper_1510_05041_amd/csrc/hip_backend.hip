// HIP implementation of the scheduler's device interface: streams by role, SDMA tile copies
// (hipMemcpy2DAsync on page-locked memory), grouped tile-step launches, events.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <map>
#include <string>
#include <vector>

#include "backend.h"

namespace blasx {

hipError_t launch_tile_steps(int dtype, bool ta, bool tb, int mode, const LaunchPack& pack, hipStream_t stream);
hipError_t launch_tile_steps_empty(int dtype, hipStream_t stream);

// Tile arena for callers that cannot allocate device memory (code under graph capture, serving loops,
// harnesses that forbid it): tile slots live in this file-scope array instead of an arena that someone
// allocated.  Every GPU the library runs on holds its own copy until the process ends.  In host code the
// array's name is only a stand-in: its device address is looked up once per device with
// hipGetSymbolAddress (backend_static_arena) and that address is what kernels and copies get.
constexpr size_t kStaticArenaBytes = (size_t)256 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticArenaBytes];

// Inverse of the nb x nb diagonal blocks of a triangular tile (the base case of the TRSM
// diagonal step; paper Eq. 1c needs A_ii^{-1}).  One wave per block, thread c solves for
// column c of the inverse by substitution.  Only the triangle is written.
template <typename T>
__global__ void trtri_blocks_kernel(const T* __restrict__ tri, int ld_tri, T* __restrict__ inv, int ld_inv, int n,
                                    int nb, int lower, int unit) {
    __shared__ double L[32][33];
    __shared__ double X[32][33];
    const int o = blockIdx.x * nb;
    const int bs = min(nb, n - o);
    const int c = threadIdx.x;
    for (int idx = threadIdx.x; idx < bs * bs; idx += blockDim.x) {
        const int r = idx % bs, q = idx / bs;
        double v = 0.0;
        if (r == q) v = unit ? 1.0 : (double)tri[(size_t)(o + r) + (size_t)(o + q) * ld_tri];
        else if (lower ? (r > q) : (r < q)) v = (double)tri[(size_t)(o + r) + (size_t)(o + q) * ld_tri];
        L[r][q] = v;
    }
    __syncthreads();
    if (c < bs) {
        X[c][c] = 1.0 / L[c][c];
        if (lower) {
            for (int r = c + 1; r < bs; ++r) {
                double s = 0.0;
                for (int q = c; q < r; ++q) s += L[r][q] * X[q][c];
                X[r][c] = -s / L[r][r];
            }
            for (int r = c; r < bs; ++r) inv[(size_t)(o + r) + (size_t)(o + c) * ld_inv] = (T)X[r][c];
        } else {
            for (int r = c - 1; r >= 0; --r) {
                double s = 0.0;
                for (int q = r + 1; q <= c; ++q) s += L[r][q] * X[q][c];
                X[r][c] = -s / L[r][r];
            }
            for (int r = 0; r <= c; ++r) inv[(size_t)(o + r) + (size_t)(o + c) * ld_inv] = (T)X[r][c];
        }
    }
}

// The full symmetric tile from its stored triangle (SYMM diagonal tiles, paper Eq. 1f): element
// (r, c) outside the stored triangle is the stored element (c, r).  32 x 32 blocks through LDS so
// that both the reads and the writes are coalesced.
template <typename T>
__global__ void symmetrize_kernel(const T* __restrict__ src, int ld_src, T* __restrict__ dst, int ld_dst, int n, int lower) {
    __shared__ T blk[32][33];
    const int br = blockIdx.x * 32, bc = blockIdx.y * 32;
    // block (br, bc) of dst comes from block (br, bc) of src when that block is in the stored
    // triangle, else from block (bc, br) transposed; diagonal blocks mix both element by element
    const bool block_stored = lower ? (br >= bc) : (br <= bc);
    const int sr = block_stored ? br : bc, sc = block_stored ? bc : br;
    for (int c = threadIdx.y; c < 32; c += blockDim.y) {
        const int r = threadIdx.x;
        T v = T(0);
        if (sr + r < n && sc + c < n) {
            const int gr = sr + r, gc = sc + c;
            const bool elem_stored = lower ? (gr >= gc) : (gr <= gc);
            if (elem_stored) v = src[(size_t)gr + (size_t)gc * ld_src];
        }
        blk[c][r] = v;          // blk[c][r] = stored (sr + r, sc + c), zero where not stored
    }
    __syncthreads();
    for (int c = threadIdx.y; c < 32; c += blockDim.y) {
        const int r = threadIdx.x;
        const int gr = br + r, gc = bc + c;
        if (gr >= n || gc >= n) continue;
        T v;
        if (br != bc) {
            v = block_stored ? blk[c][r] : blk[r][c];
        } else {
            const bool elem_stored = lower ? (gr >= gc) : (gr <= gc);
            v = elem_stored ? blk[c][r] : blk[r][c];
        }
        dst[(size_t)gr + (size_t)gc * ld_dst] = v;
    }
}

// dst = src^T through 32 x 32 LDS blocks (reads and writes both coalesced).
template <typename T>
__global__ void transpose_kernel(const T* __restrict__ src, int ld_src, int rows, int cols, T* __restrict__ dst, int ld_dst) {
    __shared__ T blk[32][33];
    const int br = blockIdx.x * 32, bc = blockIdx.y * 32;     // block origin in src
    for (int c = threadIdx.y; c < 32; c += blockDim.y) {
        const int r = threadIdx.x;
        if (br + r < rows && bc + c < cols) blk[c][r] = src[(size_t)(br + r) + (size_t)(bc + c) * ld_src];
    }
    __syncthreads();
    for (int c = threadIdx.y; c < 32; c += blockDim.y) {
        const int r = threadIdx.x;                             // dst row = src column bc + r, dst column = src row br + c
        if (bc + r < cols && br + c < rows) dst[(size_t)(bc + r) + (size_t)(br + c) * ld_dst] = blk[r][c];
    }
}

// Zeroes `height` runs of `width` 4-byte words, `pitch` words apart.
__global__ void fill_zero_kernel(uint32_t* __restrict__ p, size_t pitch, size_t width, size_t height) {
    const size_t total = width * height;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (size_t)gridDim.x * blockDim.x)
        p[(q / width) * pitch + q % width] = 0u;
}

#define HB_CHECK(call)                                   \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            err_ = std::string(#call) + ": " + hipGetErrorString(e_); \
            return 1;                                    \
        }                                                \
    } while (0)

class HipBackend : public Backend {
public:
    HipBackend() {}
    ~HipBackend() override {
        for (hipEvent_t e : events_) (void)hipEventDestroy(e);
        for (size_t s = 0; s < streams_.size(); ++s)
            if (own_stream_[s]) (void)hipStreamDestroy(streams_[s]);
    }

    int init(void* arena, size_t bytes, void* const* streams, int nstreams) {
        if (nstreams < 2 || nstreams > 4) {
            err_ = "nstreams must be 2..4";
            return 1;
        }
        if (arena) {
            arena_ = static_cast<char*>(arena);
        } else {
            // An arena the library allocates itself is kept for the next init on the device and
            // freed by backend_release_device_memory() only: while the driver clears freed device
            // memory, outbound copies run at half their rate (measured: 29.7 instead of 53.6 GB/s
            // for 0.3 s after 8 GiB were freed, for 1.5 s after 48 GiB).
            int dev = 0;
            HB_CHECK(hipGetDevice(&dev));
            OwnArena& kept = own_arenas()[dev];
            if (kept.ptr && kept.bytes < bytes) {
                (void)hipFree(kept.ptr);
                kept = OwnArena();
            }
            if (!kept.ptr) {
                HB_CHECK(hipMalloc(reinterpret_cast<void**>(&kept.ptr), bytes));
                kept.bytes = bytes;
            }
            arena_ = kept.ptr;
        }
        bytes_ = bytes;
        caller_streams_ = streams != nullptr;
        for (int s = 0; s < nstreams; ++s) {
            hipStream_t st = nullptr;
            if (streams && streams[s]) st = static_cast<hipStream_t>(streams[s]);
            else HB_CHECK(own_stream(s, &st));
            streams_.push_back(st);
            own_stream_.push_back(false);
        }
        active_ = nstreams;
        return 0;
    }

    // Streams the library makes itself live as long as the process and are reused by every later
    // init on the device: which hardware queue a stream lands on depends on what was created
    // before it, and two roles sharing one queue serialise.
    hipError_t own_stream(int s, hipStream_t* out) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        std::vector<hipStream_t>& made = own_streams()[dev];
        // All four at once, each used once straight away (an event record): a stream is given its
        // hardware queue, the least loaded one, at its first use, so four streams made and first
        // used back to back get four different queues whatever the process does later.
        while ((int)made.size() < 4 || (int)made.size() <= s) {
            hipStream_t fresh = nullptr;
            e = hipStreamCreateWithFlags(&fresh, hipStreamNonBlocking);
            if (e != hipSuccess) return e;
            made.push_back(fresh);
            hipEvent_t touch;
            if (hipEventCreateWithFlags(&touch, hipEventDisableTiming) == hipSuccess) {
                (void)hipEventRecord(touch, fresh);
                (void)hipStreamSynchronize(fresh);
                (void)hipEventDestroy(touch);
            }
        }
        *out = made[s];
        return hipSuccess;
    }

    int set_num_streams(int n) override {
        if (n < 2 || n > 4) {
            err_ = "the number of streams must be 2..4";
            return 1;
        }
        if (n > (int)streams_.size()) {
            if (caller_streams_) {
                err_ = "more streams asked for than blasx_init was given";
                return 1;
            }
            for (int s = (int)streams_.size(); s < n; ++s) {
                hipStream_t st = nullptr;
                HB_CHECK(own_stream(s, &st));
                streams_.push_back(st);
                own_stream_.push_back(false);
            }
        }
        active_ = n;
        return 0;
    }

    struct OwnArena {
        char* ptr = nullptr;
        size_t bytes = 0;
    };
    static std::map<int, OwnArena>& own_arenas() {
        static std::map<int, OwnArena> m;
        return m;
    }
    static std::map<int, std::vector<hipStream_t>>& own_streams() {
        static std::map<int, std::vector<hipStream_t>> m;
        return m;
    }

    char* arena() override { return arena_; }
    size_t arena_bytes() override { return bytes_; }
    int num_streams() override { return active_; }

    hipStream_t stream(int role) {
        const int n = active_;
        if (role < n) return streams_[role];
        return streams_[STREAM_H2D];           // fewer streams: copy roles share one
    }

    int copy_h2d(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height, int s) override {
        HB_CHECK(hipMemcpy2DAsync(dst, dpitch, src, spitch, width, height, hipMemcpyHostToDevice, stream(s)));
        return 0;
    }
    int copy_d2h(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height, int s) override {
        HB_CHECK(hipMemcpy2DAsync(dst, dpitch, src, spitch, width, height, hipMemcpyDeviceToHost, stream(s)));
        return 0;
    }
    int fill_zero(void* dev, size_t pitch, size_t width, size_t height, int s) override {
        if (width == 0 || height == 0) return 0;
        const size_t words = width / 4 * height;
        const unsigned grid = (unsigned)std::min<size_t>((words + 255) / 256, 1024);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, stream(s), static_cast<uint32_t*>(dev), pitch / 4, width / 4,
                           height);
        HB_CHECK(hipGetLastError());
        return 0;
    }
    int launch(int dtype, bool ta, bool tb, int mode, const LaunchPack& pack, int s) override {
        HB_CHECK(launch_tile_steps(dtype, ta, tb, mode, pack, stream(s)));
        return 0;
    }
    int launch_trtri_blocks(int dtype, const void* tri, int ld_tri, void* inv, int ld_inv, int n, int nb, uint32_t flags,
                            int s) override {
        if (n <= 0) return 0;
        if (nb > 32) {
            err_ = "trtri block order above 32";
            return 1;
        }
        const int grid = (n + nb - 1) / nb;
        const int lower = (flags & TS_TRI_LOWER) ? 1 : 0, unit = (flags & TS_TRI_UNIT) ? 1 : 0;
        if (dtype == 0)
            hipLaunchKernelGGL(trtri_blocks_kernel<double>, dim3(grid), dim3(64), 0, stream(s), static_cast<const double*>(tri),
                               ld_tri, static_cast<double*>(inv), ld_inv, n, nb, lower, unit);
        else
            hipLaunchKernelGGL(trtri_blocks_kernel<float>, dim3(grid), dim3(64), 0, stream(s), static_cast<const float*>(tri),
                               ld_tri, static_cast<float*>(inv), ld_inv, n, nb, lower, unit);
        HB_CHECK(hipGetLastError());
        return 0;
    }

    int launch_symmetrize(int dtype, const void* src, int ld_src, void* dst, int ld_dst, int n, bool lower, int s) override {
        if (n <= 0) return 0;
        const dim3 grid((n + 31) / 32, (n + 31) / 32), block(32, 8);
        if (dtype == 0)
            hipLaunchKernelGGL(symmetrize_kernel<double>, grid, block, 0, stream(s), static_cast<const double*>(src), ld_src,
                               static_cast<double*>(dst), ld_dst, n, lower ? 1 : 0);
        else
            hipLaunchKernelGGL(symmetrize_kernel<float>, grid, block, 0, stream(s), static_cast<const float*>(src), ld_src,
                               static_cast<float*>(dst), ld_dst, n, lower ? 1 : 0);
        HB_CHECK(hipGetLastError());
        return 0;
    }

    int launch_transpose(int dtype, const void* src, int ld_src, int rows, int cols, void* dst, int ld_dst, int s) override {
        if (rows <= 0 || cols <= 0) return 0;
        const dim3 grid((rows + 31) / 32, (cols + 31) / 32), block(32, 8);
        if (dtype == 0)
            hipLaunchKernelGGL(transpose_kernel<double>, grid, block, 0, stream(s), static_cast<const double*>(src), ld_src, rows,
                               cols, static_cast<double*>(dst), ld_dst);
        else
            hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, stream(s), static_cast<const float*>(src), ld_src, rows,
                               cols, static_cast<float*>(dst), ld_dst);
        HB_CHECK(hipGetLastError());
        return 0;
    }

    int reserve_events(int n) override {
        while ((int)events_.size() < n) {
            hipEvent_t e;
            HB_CHECK(hipEventCreate(&e));
            events_.push_back(e);
            free_.push_back((int)events_.size() - 1);
        }
        fixed_events_ = true;
        return 0;
    }
    int event_create() override {
        if (!free_.empty()) {
            const int ev = free_.back();
            free_.pop_back();
            return ev;
        }
        if (fixed_events_) {
            err_ = "event pool exhausted";
            return -1;
        }
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) {
            err_ = "hipEventCreate failed";
            return -1;
        }
        events_.push_back(e);
        return (int)events_.size() - 1;
    }
    void event_destroy(int ev) override {
        if (ev >= 0) free_.push_back(ev);
    }
    int event_record(int ev, int s) override {
        HB_CHECK(hipEventRecord(events_[ev], stream(s)));
        return 0;
    }
    int stream_wait_event(int s, int ev) override {
        HB_CHECK(hipStreamWaitEvent(stream(s), events_[ev], 0));
        return 0;
    }
    bool event_done(int ev) override { return hipEventQuery(events_[ev]) == hipSuccess; }
    int event_sync(int ev) override {
        HB_CHECK(hipEventSynchronize(events_[ev]));
        return 0;
    }
    double event_elapsed_s(int a, int b) override {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, events_[a], events_[b]) != hipSuccess) return 0.0;
        return (double)ms * 1e-3;
    }
    int sync_all() override {
        for (hipStream_t s : streams_) HB_CHECK(hipStreamSynchronize(s));
        return 0;
    }
    const char* last_error() override { return err_.c_str(); }

private:
    char* arena_ = nullptr;
    size_t bytes_ = 0;
    std::vector<hipStream_t> streams_;
    int active_ = 0;                 // streams in use (set_num_streams); the others idle
    bool caller_streams_ = false;
    std::vector<bool> own_stream_;
    std::vector<hipEvent_t> events_;
    std::vector<int> free_;
    bool fixed_events_ = false;      // reserve_events() was called: no event is created after it
    std::string err_;

public:
    hipStream_t compute_stream() { return stream(STREAM_COMPUTE); }
};

Backend* make_backend(void* arena, size_t bytes, void* const* streams, int nstreams, std::string* err) {
    HipBackend* b = new HipBackend();
    if (b->init(arena, bytes, streams, nstreams)) {
        if (err) *err = b->last_error();
        delete b;
        return nullptr;
    }
    return b;
}

void* backend_host_alloc(size_t bytes) {
    void* p = nullptr;
    if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) return nullptr;
    return p;
}

int backend_host_free(void* p) { return hipHostFree(p) == hipSuccess ? 0 : 1; }

int backend_static_arena(void** ptr, size_t* bytes) {
    static std::map<int, void*> per_device;       // each GPU holds its own copy of the array at its own address
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 1;
    auto it = per_device.find(dev);
    if (it == per_device.end()) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return 1;
        it = per_device.emplace(dev, p).first;
    }
    *ptr = it->second;
    *bytes = kStaticArenaBytes;
    return 0;
}

bool backend_host_is_pinned(const void* p) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();       // plain pageable memory is reported as an error: clear it
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}

int backend_warm_kernels(Backend& be, int dtype) {
    HipBackend& hb = static_cast<HipBackend&>(be);
    if (launch_tile_steps_empty(dtype, hb.compute_stream()) != hipSuccess) return 1;
    // the padding fill as well (no words to clear: every thread finds nothing to do)
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, hb.compute_stream(), static_cast<uint32_t*>(nullptr), (size_t)0,
                       (size_t)0, (size_t)0);
    if (hipGetLastError() != hipSuccess) return 1;
    return hipStreamSynchronize(hb.compute_stream()) == hipSuccess ? 0 : 1;
}

void backend_release_device_memory() {
    for (auto& kv : HipBackend::own_arenas()) {
        if (kv.second.ptr) (void)hipFree(kv.second.ptr);
        kv.second = HipBackend::OwnArena();
    }
}

}  // namespace blasx
