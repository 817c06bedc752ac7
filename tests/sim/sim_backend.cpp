// TEST DOUBLE -- not part of the product library.
//
// A host-only stand-in for the device interface, linked with the real task builder, tile
// cache and scheduler into tests/sim/libblasx_sim.so so that the host logic can be tested
// without a GPU.  "Device memory" is a host buffer; copies, launches and event operations are
// queued per stream and executed LAZILY, in a seeded random interleaving that respects only
// what HIP guarantees (in-order streams, event waits).  A scheduler that frees or overwrites a
// tile before the work that reads it has really run, or that forgets a cross-stream wait,
// therefore produces wrong numbers here.  The product library never loads this file.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <string>
#include <vector>

#include "../../paper_1510_05041_amd/csrc/backend.h"

namespace blasx {

namespace {

struct Op {
    enum Kind { COPY, FILL, LAUNCH, TRTRI, SYMMETRIZE, TRANSPOSE, RECORD, WAIT } kind = COPY;
    // COPY (both directions are plain strided memcpy on the host)
    char* dst = nullptr;
    const char* src = nullptr;
    size_t dpitch = 0, spitch = 0, width = 0, height = 0;
    // LAUNCH
    int dtype = 0;
    bool ta = false, tb = false;
    LaunchPack pack;
    // TRTRI
    const void* tri = nullptr;
    void* inv = nullptr;
    int ld_tri = 0, ld_inv = 0, n = 0, nb = 0;
    uint32_t flags = 0;
    // RECORD / WAIT
    int ev = -1;
    uint64_t gen = 0;
};

struct Ev {
    uint64_t issued = 0, done = 0;
    double time = 0;      // simulated device clock when the latest record ran
};

std::vector<const void*> g_h2d_sources;      // host source of every inbound copy, in issue order (trace for tests)
uint64_t g_seed = 12345;
uint64_t g_ops_run = 0, g_max_pending = 0;
bool g_deadlock = false;

template <typename T>
double tri_value(const T* p, int ld, int r, int c, uint32_t f) {
    if (r == c) return (f & TS_TRI_UNIT) ? 1.0 : (double)p[(size_t)r + (size_t)c * ld];
    const bool inside = (f & TS_TRI_LOWER) ? r > c : r < c;
    return inside ? (double)p[(size_t)r + (size_t)c * ld] : 0.0;
}

// k_quantum: what the unpredicated device kernel rounds the inner dimension of a zero-padded step up to.  The
// double reads that padding too, so that a tile whose padding was not cleared gives a wrong result here as well
// (the arena starts as NaN).
template <typename T>
void run_step(const TileStep& st, int k_quantum) {
    T* C = static_cast<T*>(st.C);
    const bool ta = st.flags & TS_TRANS_A, tb = st.flags & TS_TRANS_B;
    std::vector<double> acc((size_t)st.m * st.n, 0.0);
    for (int s = 0; s < st.nseg; ++s) {
        const TileSeg& sg = st.seg[s];
        const T* A = static_cast<const T*>(sg.A);
        const T* B = static_cast<const T*>(sg.B);
        const int k_read = (st.flags & TS_PADDED) ? round_up_to(sg.k, k_quantum) : sg.k;
        for (int j = 0; j < st.n; ++j)
            for (int l = 0; l < k_read; ++l) {
                double b;
                if (sg.flags & TS_TRI_B) b = tb ? tri_value(B, st.ldb, j, l, sg.flags) : tri_value(B, st.ldb, l, j, sg.flags);
                else b = tb ? (double)B[(size_t)j + (size_t)l * st.ldb] : (double)B[(size_t)l + (size_t)j * st.ldb];
                for (int i = 0; i < st.m; ++i) {
                    double a;
                    if (sg.flags & TS_TRI_A) a = ta ? tri_value(A, st.lda, l, i, sg.flags) : tri_value(A, st.lda, i, l, sg.flags);
                    else a = ta ? (double)A[(size_t)l + (size_t)i * st.lda] : (double)A[(size_t)i + (size_t)l * st.lda];
                    acc[(size_t)i + (size_t)j * st.m] += a * b;
                }
            }
    }
    for (int j = 0; j < st.n; ++j)
        for (int i = 0; i < st.m; ++i) {
            if ((st.flags & TS_C_LOWER) && i < j) continue;
            if ((st.flags & TS_C_UPPER) && i > j) continue;
            T* p = C + (size_t)i + (size_t)j * st.ldc;
            double v = st.alpha * acc[(size_t)i + (size_t)j * st.m];
            if (st.beta != 0.0) v += st.beta * (double)*p;
            if (st.D) v += (double)static_cast<const T*>(st.D)[(size_t)i + (size_t)j * st.ldc];
            *p = (T)v;
        }
}

template <typename T>
void run_trtri(const Op& op) {
    const T* tri = static_cast<const T*>(op.tri);
    T* inv = static_cast<T*>(op.inv);
    const bool lower = op.flags & TS_TRI_LOWER;
    for (int o = 0; o < op.n; o += op.nb) {
        const int bs = std::min(op.nb, op.n - o);
        std::vector<double> L((size_t)bs * bs, 0.0), X((size_t)bs * bs, 0.0);
        for (int c = 0; c < bs; ++c)
            for (int r = 0; r < bs; ++r) L[r + (size_t)c * bs] = tri_value(tri + (size_t)o + (size_t)o * op.ld_tri, op.ld_tri, r, c, op.flags);
        for (int c = 0; c < bs; ++c) {
            // column c of the inverse: solve L x = e_c
            if (lower) {
                for (int r = c; r < bs; ++r) {
                    double s = (r == c) ? 1.0 : 0.0;
                    for (int q = c; q < r; ++q) s -= L[r + (size_t)q * bs] * X[q + (size_t)c * bs];
                    X[r + (size_t)c * bs] = s / L[r + (size_t)r * bs];
                }
                for (int r = c; r < bs; ++r) inv[(size_t)(o + r) + (size_t)(o + c) * op.ld_inv] = (T)X[r + (size_t)c * bs];
            } else {
                for (int r = c; r >= 0; --r) {
                    double s = (r == c) ? 1.0 : 0.0;
                    for (int q = r + 1; q <= c; ++q) s -= L[r + (size_t)q * bs] * X[q + (size_t)c * bs];
                    X[r + (size_t)c * bs] = s / L[r + (size_t)r * bs];
                }
                for (int r = 0; r <= c; ++r) inv[(size_t)(o + r) + (size_t)(o + c) * op.ld_inv] = (T)X[r + (size_t)c * bs];
            }
        }
    }
}

template <typename T>
void run_symmetrize(const Op& op) {
    const T* src = static_cast<const T*>(op.tri);
    T* dst = static_cast<T*>(op.inv);
    const bool lower = op.flags & TS_TRI_LOWER;
    for (int c = 0; c < op.n; ++c)
        for (int r = 0; r < op.n; ++r) {
            const bool stored = lower ? r >= c : r <= c;
            dst[(size_t)r + (size_t)c * op.ld_inv] = stored ? src[(size_t)r + (size_t)c * op.ld_tri] : src[(size_t)c + (size_t)r * op.ld_tri];
        }
}

template <typename T>
void run_transpose(const Op& op) {
    const T* src = static_cast<const T*>(op.tri);
    T* dst = static_cast<T*>(op.inv);
    for (int c = 0; c < op.nb; ++c)
        for (int r = 0; r < op.n; ++r) dst[(size_t)c + (size_t)r * op.ld_inv] = src[(size_t)r + (size_t)c * op.ld_tri];
}

class SimBackend : public Backend {
public:
    SimBackend(size_t bytes, int nstreams) : mem_(bytes, (char)0xFF), queues_(nstreams), rng_(g_seed) {}
    ~SimBackend() override { drain(); }

    char* arena() override { return mem_.data(); }
    size_t arena_bytes() override { return mem_.size(); }
    int num_streams() override { return (int)queues_.size(); }
    int set_num_streams(int n) override {
        if (n < 2 || n > 4 || !drain()) return 1;
        queues_.resize(n);
        return 0;
    }

    int copy_h2d(void* dst, size_t dp, const void* src, size_t sp, size_t w, size_t h, int s) override {
        g_h2d_sources.push_back(src);
        return copy(dst, dp, src, sp, w, h, s);
    }
    int copy_d2h(void* dst, size_t dp, const void* src, size_t sp, size_t w, size_t h, int s) override {
        return copy(dst, dp, src, sp, w, h, s);
    }
    int fill_zero(void* dev, size_t pitch, size_t width, size_t height, int s) override {
        Op op;
        op.kind = Op::FILL;
        op.dst = static_cast<char*>(dev);
        op.dpitch = pitch;
        op.width = width;
        op.height = height;
        push(s, op);
        return 0;
    }
    int launch(int dtype, bool ta, bool tb, int mode, const LaunchPack& pack, int s) override {
        // what each kernel instantiation assumes must hold for every step of its pack
        for (int q = 0; q < pack.nsteps; ++q)
            if (step_mode(pack.step[q], dtype) > mode) {
                err_ = "launch mode does not cover a step of the pack";
                return 1;
            }
        Op op;
        op.kind = Op::LAUNCH;
        op.dtype = dtype;
        op.ta = ta;
        op.tb = tb;
        op.pack = pack;
        push(s, op);
        return 0;
    }
    int launch_trtri_blocks(int dtype, const void* tri, int ld_tri, void* inv, int ld_inv, int n, int nb, uint32_t flags,
                            int s) override {
        Op op;
        op.kind = Op::TRTRI;
        op.dtype = dtype;
        op.tri = tri;
        op.inv = inv;
        op.ld_tri = ld_tri;
        op.ld_inv = ld_inv;
        op.n = n;
        op.nb = nb;
        op.flags = flags;
        push(s, op);
        return 0;
    }
    int launch_symmetrize(int dtype, const void* src, int ld_src, void* dst, int ld_dst, int n, bool lower, int s) override {
        Op op;
        op.kind = Op::SYMMETRIZE;
        op.dtype = dtype;
        op.tri = src;
        op.inv = dst;
        op.ld_tri = ld_src;
        op.ld_inv = ld_dst;
        op.n = n;
        op.flags = lower ? TS_TRI_LOWER : 0u;
        push(s, op);
        return 0;
    }
    int launch_transpose(int dtype, const void* src, int ld_src, int rows, int cols, void* dst, int ld_dst, int s) override {
        Op op;
        op.kind = Op::TRANSPOSE;
        op.dtype = dtype;
        op.tri = src;
        op.inv = dst;
        op.ld_tri = ld_src;
        op.ld_inv = ld_dst;
        op.n = rows;
        op.nb = cols;
        push(s, op);
        return 0;
    }
    int reserve_events(int n) override {
        while ((int)events_.size() < n) {
            events_.push_back(Ev());
            free_.push_back((int)events_.size() - 1);
        }
        fixed_events_ = true;
        return 0;
    }
    int event_create() override {
        if (free_.empty() && fixed_events_) {
            err_ = "event pool exhausted";
            return -1;
        }
        if (!free_.empty()) {
            const int e = free_.back();
            free_.pop_back();
            return e;
        }
        events_.push_back(Ev());
        return (int)events_.size() - 1;
    }
    void event_destroy(int ev) override {
        if (ev >= 0) free_.push_back(ev);
    }
    int event_record(int ev, int s) override {
        Op op;
        op.kind = Op::RECORD;
        op.ev = ev;
        op.gen = ++events_[ev].issued;
        push(s, op);
        return 0;
    }
    int stream_wait_event(int s, int ev) override {
        if (events_[ev].issued == 0) return 0;
        Op op;
        op.kind = Op::WAIT;
        op.ev = ev;
        op.gen = events_[ev].issued;
        push(s, op);
        return 0;
    }
    bool event_done(int ev) override {
        const uint64_t want = events_[ev].issued;
        const int n = (int)(next() % 3);
        for (int q = 0; q < n; ++q) step();
        return events_[ev].done >= want;
    }
    int event_sync(int ev) override {
        const uint64_t want = events_[ev].issued;
        while (events_[ev].done < want)
            if (!step()) {
                g_deadlock = true;
                err_ = "simulated device deadlock";
                return 1;
            }
        return 0;
    }
    double event_elapsed_s(int a, int b) override { return events_[b].time - events_[a].time; }
    int sync_all() override { return drain() ? 0 : 1; }
    const char* last_error() override { return err_.c_str(); }

private:
    int role(int s) const { return s < (int)queues_.size() ? s : STREAM_H2D; }
    void push(int s, const Op& op) {
        queues_[role(s)].push_back(op);
        uint64_t pending = 0;
        for (auto& q : queues_) pending += q.size();
        if (pending > g_max_pending) g_max_pending = pending;
    }
    int copy(void* dst, size_t dp, const void* src, size_t sp, size_t w, size_t h, int s) {
        Op op;
        op.kind = Op::COPY;
        op.dst = static_cast<char*>(dst);
        op.src = static_cast<const char*>(src);
        op.dpitch = dp;
        op.spitch = sp;
        op.width = w;
        op.height = h;
        push(s, op);
        return 0;
    }
    uint64_t next() {
        rng_ ^= rng_ << 13;
        rng_ ^= rng_ >> 7;
        rng_ ^= rng_ << 17;
        return rng_;
    }
    bool runnable(const Op& op) const { return op.kind != Op::WAIT || events_[op.ev].done >= op.gen; }
    // run the head operation of one randomly chosen stream that can make progress
    bool step() {
        std::vector<int> ready;
        for (int s = 0; s < (int)queues_.size(); ++s)
            if (!queues_[s].empty() && runnable(queues_[s].front())) ready.push_back(s);
        if (ready.empty()) return false;
        const int s = ready[next() % ready.size()];
        Op op = queues_[s].front();
        queues_[s].pop_front();
        execute(op);
        ++g_ops_run;
        return true;
    }
    bool drain() {
        for (;;) {
            bool any = false;
            for (auto& q : queues_) any = any || !q.empty();
            if (!any) return true;
            if (!step()) {
                g_deadlock = true;
                err_ = "simulated device deadlock";
                return false;
            }
        }
    }
    // The simulated device runs one operation at a time, and its clock advances with each: a
    // launch 5 us, a tile copy 2 us, a derived-tile kernel 1 us, event operations nothing.
    void execute(const Op& op) {
        clock_ += op.kind == Op::LAUNCH ? 5e-6 : op.kind == Op::COPY ? 2e-6 : (op.kind == Op::RECORD || op.kind == Op::WAIT) ? 0.0 : 1e-6;
        switch (op.kind) {
            case Op::COPY:
                for (size_t r = 0; r < op.height; ++r) std::memcpy(op.dst + r * op.dpitch, op.src + r * op.spitch, op.width);
                break;
            case Op::FILL:
                for (size_t r = 0; r < op.height; ++r) std::memset(op.dst + r * op.dpitch, 0, op.width);
                break;
            case Op::LAUNCH:
                for (int q = 0; q < op.pack.nsteps; ++q) {
                    if (op.dtype == 0) run_step<double>(op.pack.step[q], 32);
                    else run_step<float>(op.pack.step[q], 64);
                }
                break;
            case Op::TRTRI:
                if (op.dtype == 0) run_trtri<double>(op);
                else run_trtri<float>(op);
                break;
            case Op::SYMMETRIZE:
                if (op.dtype == 0) run_symmetrize<double>(op);
                else run_symmetrize<float>(op);
                break;
            case Op::TRANSPOSE:
                if (op.dtype == 0) run_transpose<double>(op);
                else run_transpose<float>(op);
                break;
            case Op::RECORD:
                if (events_[op.ev].done < op.gen) events_[op.ev].done = op.gen;
                events_[op.ev].time = clock_;
                break;
            case Op::WAIT:
                break;
        }
    }

    std::vector<char> mem_;
    std::vector<std::deque<Op>> queues_;
    std::vector<Ev> events_;
    std::vector<int> free_;
    uint64_t rng_;
    bool fixed_events_ = false;
    double clock_ = 0;
    std::string err_;
};

}  // namespace

Backend* make_backend(void* arena, size_t bytes, void* const* streams, int nstreams, std::string* err) {
    (void)arena;
    (void)streams;
    (void)err;
    return new SimBackend(bytes, nstreams);
}

// The double has no device: the "static arena" is only a size (make_backend brings its own buffer),
// every host pointer counts as page-locked, and there are no kernels to load.
int backend_static_arena(void** ptr, size_t* bytes) {
    static char token;
    *ptr = &token;
    *bytes = (size_t)8 << 20;
    return 0;
}
bool backend_host_is_pinned(const void*) { return true; }
int backend_warm_kernels(Backend&, int) { return 0; }

void* backend_host_alloc(size_t bytes) { return std::malloc(bytes); }
void backend_release_device_memory() {}

int backend_host_free(void* p) {
    std::free(p);
    return 0;
}

}  // namespace blasx

extern "C" {
// Seed of the interleaving used by the next blasx_init of the test library.
void blasx_sim_seed(uint64_t seed) { blasx::g_seed = seed ? seed : 1; }
uint64_t blasx_sim_ops_run(void) { return blasx::g_ops_run; }
uint64_t blasx_sim_max_pending(void) { return blasx::g_max_pending; }
int blasx_sim_deadlocked(void) { return blasx::g_deadlock ? 1 : 0; }
// Trace of inbound copies: host source addresses in the order the scheduler issued them.
void blasx_sim_trace_reset(void) { blasx::g_h2d_sources.clear(); }
uint64_t blasx_sim_trace_h2d(const void** out, uint64_t max) {
    const uint64_t n = blasx::g_h2d_sources.size();
    for (uint64_t q = 0; q < n && q < max; ++q) out[q] = blasx::g_h2d_sources[q];
    return n;
}
}
