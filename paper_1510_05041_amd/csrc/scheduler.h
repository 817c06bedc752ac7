// Dynamic tile scheduler for one GPU (paper Alg. 1, lines 8-25, and Sections IV.C-D).
//
// What is kept from the paper: a queue of tile tasks; a reservation station (RS) that buffers
// upcoming tasks and ranks them by expected cache hits (Eq. 2); a small set of tasks that run
// together and advance k-step by k-step so that tile copies of one step overlap kernels of
// others; operand tiles translated through the ALRU cache; reader counts that are dropped
// only once the device has finished with a tile; result tiles written back and dropped.
//
// What differs, because one 1024^3 tile step fills a quarter of an MI355X at best:
//   - the running tasks share the GPU inside ONE grouped launch per round instead of four
//     vendor-BLAS calls on four streams, and streams are specialised by role (compute,
//     inbound copies, outbound copies);
//   - the paper's per-round StreamsSynch + ReaderUpdate is replaced by an event per launch:
//     readers are released when that event has completed, the host never drains the device;
//   - up to `kchain` consecutive k-steps of a task are fused into one launch so the
//     accumulators stay in registers;
//   - when the tile cache has room for an accumulator per output tile, ALL tasks of a call run
//     at once and advance k-chunk by k-chunk (the "wide" schedule, an outer-product order):
//     a task needs a whole block row and block column of operand tiles, so a small running set
//     starves the device while those arrive, whereas the whole task set offers about ten times
//     more products per tile copied.  The host tile of C then arrives late, in a slot of its
//     own, and the task's last launch adds the accumulated partial sums to it; inbound copies
//     are issued by a cursor that runs ahead of the launch being built.  The k loop is cut into
//     rounds of kchain steps with the left-over steps first (the last round carries every
//     result tile out and must be a full one); tasks of unequal length (triangular product)
//     are sorted by length, because a launch lasts as long as its longest chain.  The
//     triangular solve runs the same way one k-tile per round (right-looking), with every
//     diagonal tile inverted before the first round; when the device bounds the call, the
//     right-hand sides of the solve and of the triangular product run as two panels some
//     rounds apart, so that the results of one leave under the kernels of the other;
//   - inbound copies carry up to `merge` tiles: whole tiles that are neighbours in a block row
//     of the host matrix and in the arena are one strided copy (the copy engine pauses between
//     copies, not inside one); the free list hands out the lowest slot and the lists of tiles
//     to fetch are sorted so that neighbours follow each other;
//   - a grouped call whose tiles all fit the cache (the link-bound sizes) fetches C for a
//     task's last launch only, like the wide schedule, and takes its tasks block row by block
//     row, so that little is left to do when the last inbound tile has landed.
#pragma once
#include <stdint.h>

#include <cstring>
#include <deque>
#include <unordered_map>
#include <vector>

#include "alru.h"
#include "backend.h"
#include "tasks.h"

namespace blasx {

struct SchedConfig {
    int group = 0;      // tasks that run together (0 in the library's settings: chosen per call)
    int kchain = 0;     // k-steps fused per launch (1..kMaxChain; 0: chosen per run)
    int depth = 6;      // launches in flight before the host waits
    int rs = 32;        // reservation-station size
    bool priority = true;   // rank the tasks of the reservation station by Eq. 2; false: queue order (for comparison)
    int wide = 11;      // let every task of a call advance together when the cache has room and every
                        // task has at least this many k-steps (see run()); 0: never
    int prefetch = 24;  // wide mode: inbound copies are started this many launches ahead of the launch being built
    int ramp = 0;       // wide mode: k-steps per task in the first round (1..kMaxChain, cut to the chain length of
                        // the run, i.e. kMaxChain = no shorter first round; 0: chosen per run, see run())
    int merge = 0;      // most whole tiles that lie side by side in a host matrix (and land in neighbouring slots) carried
                        // by one inbound copy; 1: every tile is a copy of its own; 0: as many as make 32 MiB (2 .. 8)
    bool late_c = true; // grouped schedule: fetch the host tile of C for a task's last launch only, when the cache has room
                        // for every tile of the call (see run()); false: with the task's first launch, always
    bool row_order = true;  // the same calls take their tasks block row by block row of C instead of in the queue's order
    int tail_cut = 4;   // wide mode: tile steps per launch for the last sixteen tasks of the last round (0: sixteen, as everywhere)
    int stagger_panels = 2;   // wide triangular solve: independent panels of right-hand sides that run staggered,
    int stagger_lag = 0;      // each this many rounds behind the one before; 0: chosen per call (none when the link
                            // bounds it); -1 or one panel: all right-hand sides in step
    int profile = 0;    // 1: time every launch with events; 2: also every tile copy, and dissect the call's time on the
                        // device into kernels / copies not hidden under a kernel / neither (Section V.A, time profile)
};

struct Stats {
    uint64_t calls = 0, tasks = 0, tile_steps = 0, launches = 0;
    uint64_t hits = 0, misses = 0, evictions = 0, refetches = 0;
    uint64_t copies_h2d = 0, copies_d2h = 0, bytes_h2d = 0, bytes_d2h = 0;
    uint64_t slot_waits = 0, peak_slots = 0, profiled_launches = 0, invalidations = 0;
    double flops = 0, t_total_s = 0, t_issue_s = 0, t_kernel_s = 0;
    double t_wait_s = 0;               // host blocked on the device (events, final drain)
    double t_kernel_busy_s = 0;        // profile 2: time during which at least one kernel ran (COMPT)
    double t_copy_unoverlapped_s = 0;  // profile 2: time during which a tile copy ran and no kernel did (COMM)
    double t_device_span_s = 0;        // profile 2: first device operation of a call to its last
    uint64_t steps_general = 0;        // tile steps launched in the general (bounds-checked) kernel
    uint64_t transfers_h2d = 0;        // inbound copies handed to the copy engine (one may carry several tiles)
};

class Scheduler {
public:
    // nslots tile slots of slot_bytes each start at backend.arena().
    Scheduler(Backend& be, int nslots, size_t slot_bytes, const SchedConfig& cfg, Stats& stats);
    ~Scheduler();
    // Runs the whole problem and returns after every result tile is in host memory.
    // 0 on success, else a BLASX_ERR_* value.
    int run(Problem& p);
    // The tile cache outlives run(): a later run() on the same object finds the operand tiles
    // (and tiles derived from them) of earlier ones.  The two calls below forget cached tiles
    // whose host copy has changed; both return the number of blocks dropped.
    size_t invalidate_region(const void* base, int64_t ld, int64_t rows, int64_t cols, int esize);
    size_t invalidate_all();
    void set_config(const SchedConfig& cfg);
    size_t cached_blocks() const { return cache_.blocks(); }
    int  last_run_first_chain() const { return first_chain_; }
    bool last_run_was_wide() const { return wide_; }
    int last_run_kchain() const { return kchain_; }

private:
    struct Running {
        int task = -1;
        int next_step = 0;
        int c_slot = -1;            // slot of the accumulator (of the result once the last launch is built)
        int h_slot = -1;            // wide mode: slot the host C tile is (being) copied into, or -1
        bool first = true;          // no launch issued yet (beta_first applies)
        bool c_direct = false;      // wide mode: the host C tile is (being) copied straight into c_slot
                                    // (tasks whose first launch is their last)
        bool solved = false;
        uint64_t last_pack = 0;     // id of the pack holding this task's latest chain
        bool done = false;
    };
    struct OpenPack {
        OpenPack() { std::memset(&pack, 0, sizeof(pack)); }
        LaunchPack pack;
        std::vector<Block*> blocks;     // readers to drop when the launch retires
        std::vector<int> free_slots;    // raw slots to return when the launch retires
        std::vector<int> finishing;     // indices into running_ whose last chain is in this pack
        std::vector<int> wait_slots;    // slots whose inbound copies this launch reads
        double flops = 0;
        uint64_t steps = 0;
        int mode = 0;                   // kernel instantiation: step_mode()
        bool ta = false, tb = false;
        uint64_t id = 0;
    };
    struct InFlight {
        int done_ev = -1, start_ev = -1;
        std::vector<Block*> blocks;
        std::vector<int> free_slots;
        uint64_t id = 0;
    };
    struct WriteBack {
        int ev = -1;              // event after the last outbound copy of the launch this one belongs to
        bool owns_ev = false;     // the last entry of that launch hands the event back
        int slot = -1;
        Block* block = nullptr;   // adopted result (TRSM): drop the reader instead of freeing
        TileKey key;
    };
    struct PanelState {
        std::vector<Block*> blocks;
        int remaining = 0;
        bool loaded = false;
    };

    char* slot_ptr(int slot) const { return arena_ + (size_t)slot * slot_bytes_; }
    TileKey key_of(const TileRef& t, int tag = 0) const;
    int  new_event();
    void put_event(int ev) { free_events_.push_back(ev); }

    int  fetch(const TileRef& t, Block** out);               // translate + inbound copy on a miss
    int  issue_h2d(const TileRef& t, int slot);
    int  release_held();                                     // hands the inbound copy that is being gathered to the engine
    int  fetch_sorted(std::vector<const TileRef*>& refs, bool may_evict);
    void prefetch_grouped_round();
    int  zero_padding(int slot, int rows, int cols, int stream);
    int  take_slot_blocking(int* slot);
    int  start_task(int task_index, Running* r);
    int  ensure_panel(int panel);
    int  reserve_all_panels();
    int  build_chain(int ri);
    const std::vector<uint32_t>& round_order(size_t round);
    int  prefetch_c(Running& r, const Task& t, bool may_wait);
    int  load_c_direct(Running& r, const Task& t);
    void prefetch_ahead(size_t build_pos);
    bool wide_fits(const Problem& p);
    // wide mode: first k-step of round r
    // first k-step of round r: rounds are kchain_ steps long, except that the first two may be shorter
    size_t round_begin(size_t r) const {
        return r == 0 ? 0 : r == 1 ? (size_t)first_chain_ : (size_t)(first_chain_ + second_chain_) + (r - 2) * (size_t)kchain_;
    }
    int  build_solve(int ri);
    int  get_inverse(const Task& t, Block** out);
    int  make_inverses(const Task* const* tasks, size_t count, bool prefetch_after_fetch = false);
    // wide solve: the round of a task's own schedule that global round R is (negative: its panel has not started)
    long local_round(size_t task, size_t R) const { return lag_.empty() ? (long)R : (long)R - (long)lag_[task]; }
    std::vector<const Task*> diag_tasks(const Problem& p) const;
    int  fetch_derived(const TileRef& t, int kind, Block** out);
    OpenPack& pack_for(int mode, bool ta, bool tb) { return packs_[mode][ta ? 1 : 0][tb ? 1 : 0]; }
    bool pack_is_open(uint64_t id) const;
    int  add_step(OpenPack& op, bool ta, bool tb, const TileStep& st, double flops, uint64_t nsteps);
    int  flush(OpenPack& op);
    int  flush_all();
    int  finish_task(int ri);
    int  fill_event(int slot);
    bool retire(bool block_on_oldest);
    void poll_writebacks(bool block);
    void wait_event(int ev);            // blocks the host; the time counts as waiting, not issuing
    int  profiled_copy_begin(int stream);
    int  profiled_copy_end(int stream);
    void dissect_time();
    void refill_rs();
    int  pick_from_rs();
    bool deps_started(const Task& t) const;
    int64_t priority(const Task& t) const;

    Backend& be_;
    Alru cache_;
    char* arena_;
    size_t slot_bytes_;
    SchedConfig cfg_;
    Stats& stats_;
    Problem* p_ = nullptr;
    int T_ = 0;
    // Tiles are kept zero-padded to whole macro-tiles in their slots (possible when the slot edge is a multiple
    // of the macro-tile edge): ragged tile steps can then run in the unpredicated kernel (TS_PADDED).
    bool pad_ok_ = false;
    int kchain_ = 4;                    // this run: k-steps fused per launch
    bool wide_ = false;                 // this run: all tasks advance together, C tiles arrive late
    int merge_ = 1;                     // this run: most tiles per inbound copy
    int pack_cut_ = 16;                 // a launch pack is launched when it holds this many tile steps
    bool late_c_ = false;               // this run: a task's host C tile is fetched for its last launch (wide, or grouped with room)
    size_t round_ = 0;                  // wide mode: index of the round being built
    std::vector<uint32_t> lag_;         // wide solve: rounds by which each task's panel trails the first one (empty: none)
    size_t pf_last_round_ = 0;          // wide mode: last round in which any task still has steps
    size_t pfc_pos_ = 0;                // wide mode: same for the host C tiles, which run further ahead
    size_t pf_reserve_ = 0;             // free slots that early C tiles must leave for operand tiles
    int second_chain_ = 0;              // wide mode: k-steps per task in the second round (<= kchain_)
    bool force_open_ = false;           // pick_from_rs(): ignore the bound on open panels (nothing else can run)
    int first_chain_ = 0;               // wide mode: k-steps per task in the first round (<= kchain_)
    size_t build_pos_ = 0;              // wide mode: (round * ntasks + position in the round's order) of the chain being built
    static constexpr int kOrders = 4;   // the round being built and those the two prefetch cursors are in
    std::vector<uint32_t> order_[kOrders];   // wide mode: round_order() of the latest rounds asked for
    size_t order_round_[kOrders] = {SIZE_MAX, SIZE_MAX, SIZE_MAX, SIZE_MAX};
    size_t pf_pos_ = 0;                 // wide mode: next (round * ntasks + task) whose tiles get prefetched

    std::vector<int> fill_ev_;          // per slot: event of its latest inbound copy
    std::vector<uint64_t> fill_seq_;    // per slot: number of its latest inbound copy on its stream (0: none yet)
    std::vector<int> fill_stream_;
    uint64_t h2d_issued_[4] = {0, 0, 0, 0};      // per stream role
    uint64_t compute_waited_[4] = {0, 0, 0, 0};
    int h2d_rr_ = 0;
    // An inbound copy that has not been handed to the copy engine yet: whole tiles that follow each other along a
    // block row of a host matrix and whose slots follow each other in the arena travel as one strided copy
    // (the engine leaves about 10 us between two copies, whatever their size).
    static constexpr int kMaxMerge = 8;
    struct HeldCopy {
        int stream = -1;                // -1: nothing held
        char* dst = nullptr;
        const char* src = nullptr;
        size_t spitch = 0;              // bytes between columns in the host matrix
        int ntiles = 0;
        int slots[kMaxMerge];
    } held_;

    size_t next_task_ = 0;
    std::vector<int> rs_;               // task indices waiting in the reservation station
    std::vector<int64_t> rs_prio_;      // their priorities (Eq. 2), refreshed when tasks enter
    bool rs_dirty_ = true;
    std::vector<Running> running_;
    std::vector<char> task_started_, task_issued_;   // per task
    std::vector<uint64_t> task_final_pack_;          // pack id of the launch that finishes it
    std::vector<PanelState> panels_;
    OpenPack packs_[3][2][2];           // open launch packs, one per kernel instantiation (mode, transA, transB)
    uint64_t next_pack_id_ = 1;
    std::deque<InFlight> inflight_;
    std::deque<WriteBack> writebacks_;
    std::unordered_map<TileKey, int, TileKeyHash> pending_wb_;   // host tile -> event of its outbound copy
    std::vector<int> free_events_;
    double t_wait_ = 0;                 // this run: host time spent blocked on the device
    // profile 2: event pairs around every launch and every tile copy of this run, and the event all times count from
    struct Interval { int begin_ev, end_ev; };
    std::vector<Interval> kernel_iv_, copy_iv_;
    int base_ev_ = -1;
    int err_ = 0;
};

}  // namespace blasx
