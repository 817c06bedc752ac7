#include "scheduler.h"

#include <algorithm>
#include <chrono>
#include <cstring>
#include <unordered_set>

#include "../../include/blasx.h"

namespace blasx {

namespace {
double now_s() {
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
constexpr int kTrtriBlock = 32;   // order of the diagonal blocks inverted directly
// grouped schedule with room: operand tiles are asked for this many launches per task ahead, so that a task's tiles
// of a block row come in as few copies
constexpr int kHintChains = 4;
// cache-key tags of tiles derived on the device (1..4 are the inverses of triangular diagonal tiles)
constexpr int kDerivedSymUpper = 5, kDerivedSymLower = 6, kDerivedTranspose = 7;
}  // namespace

#define BX_TRY(expr)                      \
    do {                                  \
        const int rc_ = (expr);           \
        if (rc_ != 0) return rc_;         \
    } while (0)

Scheduler::Scheduler(Backend& be, int nslots, size_t slot_bytes, const SchedConfig& cfg, Stats& stats)
    : be_(be), cache_(nslots), arena_(be.arena()), slot_bytes_(slot_bytes), cfg_(cfg), stats_(stats) {
    fill_ev_.assign(nslots, -1);
    fill_seq_.assign(nslots, 0);
    fill_stream_.assign(nslots, STREAM_H2D);
    set_config(cfg);
    for (int q = 0; q < 3; ++q)
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b) packs_[q][a][b].mode = q;
}

void Scheduler::set_config(const SchedConfig& cfg) {
    cfg_ = cfg;
    cfg_.kchain = std::max(0, std::min(cfg_.kchain, kMaxChain));   // 0: chosen per run
    kchain_ = cfg_.kchain ? cfg_.kchain : 4;
    cfg_.group = std::max(1, cfg_.group);
    cfg_.depth = std::max(1, cfg_.depth);
    cfg_.rs = std::max(cfg_.rs, cfg_.group);
}

size_t Scheduler::invalidate_region(const void* base, int64_t ld, int64_t rows, int64_t cols, int esize) {
    const size_t n = cache_.invalidate_region(base, ld, rows, cols, esize);
    stats_.invalidations += n;
    return n;
}

size_t Scheduler::invalidate_all() {
    const size_t n = cache_.invalidate_all();
    stats_.invalidations += n;
    return n;
}

Scheduler::~Scheduler() {
    for (int ev : fill_ev_)
        if (ev >= 0) be_.event_destroy(ev);
    for (int ev : free_events_) be_.event_destroy(ev);
}

// Event whose completion implies that the latest inbound copy into `slot` has landed.  Every
// copy gets an event of its own (re-recorded when the slot is filled again): measured on the
// copy engines an event record costs under 1 us next to a 150 us tile copy, while an event shared
// by several copies would make a launch wait for copies that were only prefetched for later ones.
// A copy that is still being gathered goes out first, so that the event of every slot that has been
// given a copy has been recorded when somebody orders work after it.
int Scheduler::fill_event(int slot) {
    if (held_.stream >= 0 && release_held()) err_ = BLASX_ERR_DEVICE;
    return fill_ev_[slot];
}

TileKey Scheduler::key_of(const TileRef& t, int tag) const {
    TileKey k;
    k.host = t.host;
    k.ld = t.ld;
    k.rows = t.rows;
    k.cols = t.cols;
    k.esize = (int32_t)p_->esize;
    k.tag = tag;
    return k;
}

int Scheduler::new_event() {
    if (!free_events_.empty()) {
        const int ev = free_events_.back();
        free_events_.pop_back();
        return ev;
    }
    return be_.event_create();
}

// ---------------------------------------------------------------- completion tracking ----

// Alg. 1 "ReaderUpdate": drop the readers of every launch the device has finished.  The
// paper does this after a full StreamsSynch; here one event per launch tells the same thing
// without draining the streams.
void Scheduler::wait_event(int ev) {
    if (held_.stream >= 0 && release_held()) err_ = BLASX_ERR_DEVICE;    // the host is about to sleep: nothing is held back
    const double t = now_s();
    be_.event_sync(ev);
    t_wait_ += now_s() - t;
}

bool Scheduler::retire(bool block_on_oldest) {
    bool any = false;
    while (!inflight_.empty()) {
        InFlight& f = inflight_.front();
        if (!be_.event_done(f.done_ev)) {
            if (!block_on_oldest) break;
            wait_event(f.done_ev);
        }
        block_on_oldest = false;
        bool keep_events = false;
        if (f.start_ev >= 0) {
            stats_.t_kernel_s += be_.event_elapsed_s(f.start_ev, f.done_ev);
            ++stats_.profiled_launches;
            if (cfg_.profile >= 2) {
                kernel_iv_.push_back(Interval{f.start_ev, f.done_ev});   // handed back by dissect_time()
                keep_events = true;
            } else {
                put_event(f.start_ev);
            }
        }
        for (Block* b : f.blocks) cache_.release(b);
        for (int s : f.free_slots) cache_.give_slot(s);
        if (!keep_events) put_event(f.done_ev);
        inflight_.pop_front();
        any = true;
    }
    return any;
}

// Result tiles whose outbound copy has landed: their slot is free again (or, for TRSM, the
// adopted cache block loses the reader that protected it during the copy).
void Scheduler::poll_writebacks(bool block) {
    while (!writebacks_.empty()) {
        WriteBack& w = writebacks_.front();
        if (!be_.event_done(w.ev)) {
            if (!block) break;
            wait_event(w.ev);
        }
        if (w.block) {
            cache_.release(w.block);
            auto it = pending_wb_.find(w.key);
            if (it != pending_wb_.end() && it->second == w.ev) pending_wb_.erase(it);
        } else {
            cache_.give_slot(w.slot);
        }
        if (w.owns_ev) put_event(w.ev);
        writebacks_.pop_front();
    }
}

int Scheduler::take_slot_blocking(int* slot) {
    for (;;) {
        const int s = cache_.take_slot();
        if (s >= 0) {
            // fill_seq_ / fill_stream_ of the slot are kept: an inbound copy issued for its previous
            // owner may still be in flight, and whoever writes the slot next must be ordered after it
            *slot = s;
            return 0;
        }
        ++stats_.slot_waits;
        BX_TRY(flush_all());
        if (!inflight_.empty()) {
            retire(true);
        } else if (!writebacks_.empty()) {
            poll_writebacks(true);
        } else {
            return BLASX_ERR_ARENA_TOO_SMALL;
        }
        poll_writebacks(false);
    }
}

// ---------------------------------------------------------------- tile movement ----------

// profile 2: an event before and one after every tile copy, on the copy's own stream
int Scheduler::profiled_copy_begin(int stream) {
    if (cfg_.profile < 2) return 0;
    const int ev = new_event();
    if (ev < 0 || be_.event_record(ev, stream)) return BLASX_ERR_DEVICE;
    copy_iv_.push_back(Interval{ev, -1});
    return 0;
}

int Scheduler::profiled_copy_end(int stream) {
    if (cfg_.profile < 2) return 0;
    const int ev = new_event();
    if (ev < 0 || be_.event_record(ev, stream)) return BLASX_ERR_DEVICE;
    copy_iv_.back().end_ev = ev;
    return 0;
}

// Section V.A dissects a run into computation, communication that no computation hides, and the
// rest.  From the event pairs of this run: the time covered by kernels, and the time covered by
// tile copies but by no kernel.  Every event has completed when this runs.
void Scheduler::dissect_time() {
    if (base_ev_ < 0) return;
    auto spans = [&](std::vector<Interval>& iv) {
        std::vector<std::pair<double, double>> out;
        for (const Interval& q : iv) {
            if (q.end_ev >= 0) {
                const double b = be_.event_elapsed_s(base_ev_, q.begin_ev), e = be_.event_elapsed_s(base_ev_, q.end_ev);
                if (e > b) out.emplace_back(b, e);
                put_event(q.end_ev);
            }
            put_event(q.begin_ev);
        }
        iv.clear();
        std::sort(out.begin(), out.end());
        std::vector<std::pair<double, double>> merged;      // disjoint, ascending
        for (const auto& q : out) {
            if (!merged.empty() && q.first <= merged.back().second) merged.back().second = std::max(merged.back().second, q.second);
            else merged.push_back(q);
        }
        return merged;
    };
    const auto kern = spans(kernel_iv_), copy = spans(copy_iv_);
    double busy = 0, hidden = 0, copying = 0, first = 1e300, last = 0;
    for (const auto& q : kern) busy += q.second - q.first;
    size_t k = 0;
    for (const auto& c : copy) {
        copying += c.second - c.first;
        while (k < kern.size() && kern[k].second <= c.first) ++k;
        for (size_t q = k; q < kern.size() && kern[q].first < c.second; ++q)
            hidden += std::min(c.second, kern[q].second) - std::max(c.first, kern[q].first);
    }
    for (const auto* v : {&kern, &copy})
        if (!v->empty()) {
            first = std::min(first, v->front().first);
            last = std::max(last, v->back().second);
        }
    stats_.t_kernel_busy_s += busy;
    stats_.t_copy_unoverlapped_s += copying - hidden;
    if (last > first) stats_.t_device_span_s += last - first;
    put_event(base_ev_);
    base_ev_ = -1;
}

// Clears what lies between a tile's true extent and the next multiples of the macro-tile edge in its slot
// (the columns beyond `cols` as whole columns of the slot, then the rows beyond `rows` of the true columns),
// on `stream`, so that the unpredicated kernel can read the tile on its padded extent.
int Scheduler::zero_padding(int slot, int rows, int cols, int stream) {
    if (!pad_ok_) return 0;
    const size_t es = p_->esize;
    const int rows_pad = round_up_to(rows, kBM), cols_pad = round_up_to(cols, kBN);
    char* base = slot_ptr(slot);
    if (cols_pad > cols &&
        be_.fill_zero(base + (size_t)cols * T_ * es, (size_t)T_ * es, (size_t)(cols_pad - cols) * T_ * es, 1, stream))
        return BLASX_ERR_DEVICE;
    if (rows_pad > rows && cols > 0 &&
        be_.fill_zero(base + (size_t)rows * es, (size_t)T_ * es, (size_t)(rows_pad - rows) * es, (size_t)cols, stream))
        return BLASX_ERR_DEVICE;
    return 0;
}

// Hands the copy that issue_h2d() has been gathering to the copy engine, and records the event of every slot it fills.
int Scheduler::release_held() {
    if (held_.stream < 0) return 0;
    const int stream = held_.stream;
    held_.stream = -1;
    const size_t es = p_->esize;
    BX_TRY(profiled_copy_begin(stream));
    if (be_.copy_h2d(held_.dst, (size_t)T_ * es, held_.src, held_.spitch, (size_t)T_ * es, (size_t)T_ * held_.ntiles, stream))
        return BLASX_ERR_DEVICE;
    BX_TRY(profiled_copy_end(stream));
    for (int q = 0; q < held_.ntiles; ++q) {
        const int slot = held_.slots[q];
        if (fill_ev_[slot] < 0) fill_ev_[slot] = be_.event_create();
        if (be_.event_record(fill_ev_[slot], stream)) return BLASX_ERR_DEVICE;
    }
    ++stats_.transfers_h2d;
    return 0;
}

// Starts the inbound copy of a host tile into `slot`.  A whole tile is not handed to the copy engine at once: if the
// next tile asked for is its right-hand neighbour in the host matrix and goes to the next slot of the arena, the two
// (up to `merge` of them) are one strided copy -- the columns of the second tile follow those of the first at the same
// pitch on both sides.  The copy goes out when a tile that does not continue it is asked for, when anybody needs the
// event of one of its slots, when a launch is issued and before the host blocks.
int Scheduler::issue_h2d(const TileRef& t, int slot) {
    const size_t es = p_->esize;
    const size_t spitch = (size_t)t.ld * es;
    const bool whole = merge_ > 1 && t.rows == T_ && t.cols == T_;
    if (held_.stream >= 0) {
        // (a slot whose previous copy went through the other stream needs an ordering wait first: not merged)
        if (whole && held_.ntiles < merge_ && spitch == held_.spitch &&
            t.host == held_.src + (size_t)held_.ntiles * T_ * spitch &&
            slot_ptr(slot) == held_.dst + (size_t)held_.ntiles * T_ * T_ * es &&
            (fill_seq_[slot] == 0 || fill_stream_[slot] == held_.stream)) {
            held_.slots[held_.ntiles++] = slot;
            fill_seq_[slot] = ++h2d_issued_[held_.stream];
            fill_stream_[slot] = held_.stream;
            ++stats_.copies_h2d;
            stats_.bytes_h2d += (uint64_t)t.rows * t.cols * es;
            return 0;
        }
        BX_TRY(release_held());
    }
    int stream = STREAM_H2D;
    if (be_.num_streams() >= 4) {
        stream = (h2d_rr_++ & 1) ? STREAM_H2D_B : STREAM_H2D;
    }
    // A slot can change owner while a copy for its previous owner is still queued on the other
    // inbound stream (a block that was evicted before any launch read it): order the two copies.
    if (fill_seq_[slot] != 0 && fill_stream_[slot] != stream) {
        if (be_.stream_wait_event(stream, fill_event(slot))) return BLASX_ERR_DEVICE;
    }
    if (whole) {
        held_.stream = stream;
        held_.dst = slot_ptr(slot);
        held_.src = t.host;
        held_.spitch = spitch;
        held_.ntiles = 1;
        held_.slots[0] = slot;
    } else {
        BX_TRY(profiled_copy_begin(stream));
        if (be_.copy_h2d(slot_ptr(slot), (size_t)T_ * es, t.host, spitch, (size_t)t.rows * es, (size_t)t.cols, stream))
            return BLASX_ERR_DEVICE;
        BX_TRY(profiled_copy_end(stream));
        BX_TRY(zero_padding(slot, (int)t.rows, (int)t.cols, stream));     // before the fill event: consumers see the padded tile
        if (fill_ev_[slot] < 0) fill_ev_[slot] = be_.event_create();
        if (be_.event_record(fill_ev_[slot], stream)) return BLASX_ERR_DEVICE;
        ++stats_.transfers_h2d;
    }
    fill_seq_[slot] = ++h2d_issued_[stream];
    fill_stream_[slot] = stream;
    ++stats_.copies_h2d;
    stats_.bytes_h2d += (uint64_t)t.rows * t.cols * es;
    return 0;
}

// Inbound copies that are wanted soon, started in an order in which tiles that lie side by side in a host matrix
// follow each other (so that issue_h2d() can carry them in one copy): by leading dimension, then by the position of
// the tile's block row within a column, then by address.  Tiles already cached are skipped.  Without may_evict only
// free slots are used.  Returns what fetch() returns for the first tile that could not be started (-1: no slot).
int Scheduler::fetch_sorted(std::vector<const TileRef*>& refs, bool may_evict) {
    const size_t es = p_->esize;
    auto row_of = [es](const TileRef* r) { return r->ld > 0 ? (uintptr_t)r->host % ((uintptr_t)r->ld * es) : (uintptr_t)0; };
    std::sort(refs.begin(), refs.end(), [&](const TileRef* x, const TileRef* y) {
        if (x->ld != y->ld) return x->ld < y->ld;
        const uintptr_t rx = row_of(x), ry = row_of(y);
        if (rx != ry) return rx < ry;
        return x->host < y->host;
    });
    const TileRef* prev = nullptr;
    for (const TileRef* ref : refs) {
        if (prev && prev->host == ref->host && prev->ld == ref->ld && prev->rows == ref->rows && prev->cols == ref->cols) continue;
        prev = ref;
        const Block* have = cache_.find(key_of(*ref));
        if (have && !have->pending) continue;
        if (!may_evict && !have && cache_.used_slots() >= cache_.nslots()) return -1;
        Block* b = nullptr;
        const int rc = fetch(*ref, &b);
        if (rc) return rc;
    }
    return 0;
}

// Alg. 1 lines 22-23 (tile = CCP(&tile)): translate a host tile to its device copy, starting
// the inbound copy when it is not cached.  -1: no slot could be found right now.
int Scheduler::fetch(const TileRef& t, Block** out) {
    const TileKey key = key_of(t);
    bool hit = false;
    Block* b = cache_.translate(key, &hit);
    if (!b) return -1;
    if (!hit || b->pending) {
        b->pending = false;
        auto it = pending_wb_.find(key);
        if (it != pending_wb_.end()) {
            // the host copy of this tile is still being written by an outbound copy
            if (be_.stream_wait_event(STREAM_H2D, it->second)) return BLASX_ERR_DEVICE;
            if (be_.num_streams() >= 4 && be_.stream_wait_event(STREAM_H2D_B, it->second)) return BLASX_ERR_DEVICE;
        }
        const int rc = issue_h2d(t, b->slot);
        if (rc) return rc;
    }
    *out = b;
    return 0;
}

// TRMM: fetch and pin the original tiles of a panel before its first task starts.
int Scheduler::ensure_panel(int panel) {
    PanelState& ps = panels_[panel];
    if (ps.loaded) return 0;
    const Panel& pn = p_->panels[panel];
    for (const TileRef& t : pn.tiles) {
        Block* b = nullptr;
        for (;;) {
            // Wide schedule: every panel is entered at once, so the tiles are only given their
            // slots here (they must never be evicted and fetched again once results overwrite the
            // host matrix); each is copied in when its first reader, or the prefetch cursor, gets to it.
            int rc = 0;
            if (wide_) {
                bool hit = false;
                b = cache_.translate(key_of(t), &hit);
                if (!b) rc = -1;
                else if (!hit) b->pending = true;
            } else {
                rc = fetch(t, &b);
            }
            if (rc == 0) break;
            if (rc > 0) return rc;
            ++stats_.slot_waits;
            BX_TRY(flush_all());
            if (!inflight_.empty()) retire(true);
            else if (!writebacks_.empty()) poll_writebacks(true);
            else return BLASX_ERR_ARENA_TOO_SMALL;
        }
        cache_.acquire(b);
        ps.blocks.push_back(b);
    }
    ps.loaded = true;
    return 0;
}

// Wide TRMM: every panel is entered at once, so all their tiles get their slots here in one pass, block row by block
// row of the matrix across the panels: tiles that are neighbours in the host matrix then sit in neighbouring slots and
// can share an inbound copy (panel by panel, the neighbours of a tile would be a whole panel of slots away).
int Scheduler::reserve_all_panels() {
    struct Want { const TileRef* ref; int panel; };
    std::vector<Want> all;
    for (size_t q = 0; q < p_->panels.size(); ++q) {
        if (panels_[q].loaded) continue;
        for (const TileRef& t : p_->panels[q].tiles) all.push_back(Want{&t, (int)q});
    }
    const size_t es = p_->esize;
    auto row_of = [es](const TileRef* r) { return r->ld > 0 ? (uintptr_t)r->host % ((uintptr_t)r->ld * es) : (uintptr_t)0; };
    std::stable_sort(all.begin(), all.end(), [&](const Want& x, const Want& y) {
        const uintptr_t rx = row_of(x.ref), ry = row_of(y.ref);
        return rx != ry ? rx < ry : x.ref->host < y.ref->host;
    });
    for (const Want& w : all) {
        bool hit = false;
        Block* b = cache_.translate(key_of(*w.ref), &hit);
        if (!b) return BLASX_ERR_ARENA_TOO_SMALL;        // wide_fits() has counted them
        if (!hit) b->pending = true;
        cache_.acquire(b);
        panels_[w.panel].blocks.push_back(b);
    }
    for (size_t q = 0; q < p_->panels.size(); ++q) panels_[q].loaded = true;
    return 0;
}

// ---------------------------------------------------------------- reservation station ----

void Scheduler::refill_rs() {
    const size_t ntasks = p_->tasks.size();
    while ((int)rs_.size() < cfg_.rs && next_task_ < ntasks) {
        rs_.push_back((int)next_task_++);
        rs_dirty_ = true;
    }
}

bool Scheduler::deps_started(const Task& t) const {
    for (const StepSpec& s : t.steps)
        if (s.dep >= 0 && !task_started_[s.dep]) return false;
    return true;
}

// Eq. 2: priority = sum over the task's steps of f(A_ik) + f(B_kj), f = 2 for a tile that is in
// the (single-level) cache and 0 otherwise.
int64_t Scheduler::priority(const Task& t) const {
    int64_t pr = 0;
    if (!cfg_.priority) return 0;
    for (const StepSpec& s : t.steps) {
        if (cache_.find(key_of(s.a))) pr += 2;
        if (cache_.find(key_of(s.b))) pr += 2;
    }
    return pr;
}

// Highest-priority task of the RS whose producers have all started; ties go to queue order.
// Priorities are refreshed when new tasks have entered the RS (Section IV.C).
int Scheduler::pick_from_rs() {
    if (rs_.empty()) return -1;
    if (rs_dirty_) {
        rs_prio_.resize(rs_.size());
        for (size_t q = 0; q < rs_.size(); ++q) rs_prio_[q] = priority(p_->tasks[rs_[q]]);
        rs_dirty_ = false;
    }
    // TRMM: a panel's original tiles stay pinned until the last of its tasks has finished, so the
    // number of panels entered and not yet finished is bounded by what half the cache holds; a
    // task of a further panel waits until one is finished (tasks of open panels are preferred).
    size_t open_panels = 0, panel_tiles = 1;
    for (size_t q = 0; q < panels_.size(); ++q) {
        open_panels += panels_[q].loaded && panels_[q].remaining > 0 ? 1 : 0;
        panel_tiles = std::max(panel_tiles, p_->panels[q].tiles.size());
    }
    const bool may_open = force_open_ || open_panels == 0 || (open_panels + 1) * panel_tiles <= (size_t)cache_.nslots() / 2;
    int best = -1;
    for (size_t q = 0; q < rs_.size(); ++q) {
        const Task& t = p_->tasks[rs_[q]];
        if (!deps_started(t)) continue;
        if (t.panel >= 0 && !panels_[t.panel].loaded && !may_open) continue;
        if (best < 0 || rs_prio_[q] > rs_prio_[best]) best = (int)q;
    }
    if (best < 0) return -1;
    const int task = rs_[best];
    rs_.erase(rs_.begin() + best);
    rs_prio_.erase(rs_prio_.begin() + best);
    return task;
}

// ---------------------------------------------------------------- launches ---------------

int Scheduler::add_step(OpenPack& op, bool ta, bool tb, const TileStep& st, double flops, uint64_t nsteps) {
    if (op.pack.nsteps > 0 && (op.ta != ta || op.tb != tb)) BX_TRY(flush(op));
    // A launch is cut at a multiple of 8 steps: 8 whole-tile steps of 64 macro-tiles fill the 512
    // workgroup slots of the chip once, so multiples of 8 leave no partial wave of workgroups.
    if (op.pack.nsteps >= pack_cut_) BX_TRY(flush(op));
    if (op.pack.nsteps == 0) {
        op.ta = ta;
        op.tb = tb;
        op.id = next_pack_id_++;
        op.pack.total_wg = 0;
    }
    TileStep& dst = op.pack.step[op.pack.nsteps++];
    dst = st;
    dst.wg_begin = op.pack.total_wg;
    op.pack.total_wg += macro_tiles(st.m, st.n, st.flags);
    op.flops += flops;
    op.steps += nsteps;
    return 0;
}

int Scheduler::flush(OpenPack& op) {
    if (op.pack.nsteps == 0) return 0;
    BX_TRY(release_held());
    // Make the compute stream wait for the inbound copies this launch reads: one wait per
    // copy stream is enough, on the youngest copy (streams are in order).
    for (int stream : {(int)STREAM_H2D, (int)STREAM_H2D_B}) {
        int best = -1;
        for (int s : op.wait_slots)
            if (fill_stream_[s] == stream && fill_seq_[s] > compute_waited_[stream] &&
                (best < 0 || fill_seq_[s] > fill_seq_[best]))
                best = s;
        if (best >= 0) {
            if (be_.stream_wait_event(STREAM_COMPUTE, fill_event(best))) return BLASX_ERR_DEVICE;
            compute_waited_[stream] = fill_seq_[best];
        }
    }
    InFlight f;
    f.id = op.id;
    if (cfg_.profile) {
        f.start_ev = new_event();
        if (be_.event_record(f.start_ev, STREAM_COMPUTE)) return BLASX_ERR_DEVICE;
    }
    if (be_.launch(p_->dtype, op.ta, op.tb, op.mode, op.pack, STREAM_COMPUTE)) return BLASX_ERR_DEVICE;
    f.done_ev = new_event();
    if (be_.event_record(f.done_ev, STREAM_COMPUTE)) return BLASX_ERR_DEVICE;
    f.blocks.swap(op.blocks);
    f.free_slots.swap(op.free_slots);
    ++stats_.launches;
    stats_.tile_steps += op.steps;
    if (op.mode == 2) stats_.steps_general += op.steps;
    stats_.flops += op.flops;
    const int done_ev = f.done_ev;
    inflight_.push_back(std::move(f));
    std::vector<int> finishing;
    finishing.swap(op.finishing);
    op.pack.nsteps = 0;
    op.pack.total_wg = 0;
    op.wait_slots.clear();
    op.flops = 0;
    op.steps = 0;
    if (!finishing.empty()) {
        // the write-backs of one launch: one wait before them, one event after them
        const int d2h = be_.num_streams() >= 3 ? STREAM_D2H : STREAM_H2D;
        if (be_.stream_wait_event(d2h, done_ev)) return BLASX_ERR_DEVICE;
        const size_t first = writebacks_.size();
        for (int ri : finishing) BX_TRY(finish_task(ri));
        const int ev = new_event();
        if (be_.event_record(ev, d2h)) return BLASX_ERR_DEVICE;
        for (size_t q = first; q < writebacks_.size(); ++q) {
            writebacks_[q].ev = ev;
            if (writebacks_[q].block) pending_wb_[writebacks_[q].key] = ev;
        }
        writebacks_.back().owns_ev = true;
    }
    // bound the host's run-ahead: at most `depth` launches in flight
    while ((int)inflight_.size() > cfg_.depth) retire(true);
    return 0;
}

// Whether the launch pack with this id is still being filled (its steps have not been launched).  Packs of
// different kernel instantiations are open side by side and are launched in no particular order of their
// ids -- a full one goes out while an older one of another kind is still open -- so "launched" cannot be
// told from the largest id launched so far.
bool Scheduler::pack_is_open(uint64_t id) const {
    for (int q = 0; q < 3; ++q)
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b)
                if (packs_[q][a][b].pack.nsteps > 0 && packs_[q][a][b].id == id) return true;
    return false;
}

int Scheduler::flush_all() {
    BX_TRY(release_held());
    for (int q = 0; q < 3; ++q)
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b) BX_TRY(flush(packs_[q][a][b]));
    return 0;
}

// The last launch of a task has been issued: write the tile back to the host matrix once that
// launch is done, and let go of it (the paper's ephemeral M state: written back, then invalid).
int Scheduler::finish_task(int ri) {
    Running& r = running_[ri];
    const Task& t = p_->tasks[r.task];
    const size_t es = p_->esize;
    const int d2h = be_.num_streams() >= 3 ? STREAM_D2H : STREAM_H2D;
    if (t.panel >= 0) {
        // In-place update: the original of the tile this result overwrites is an operand of other
        // tasks of the panel.  It is pinned in the cache; it must have been read from the host
        // before the outbound copy lands there.
        TileRef own;
        own.host = t.c_host;
        own.ld = p_->ldc;
        own.rows = t.m;
        own.cols = t.n;
        Block* b = nullptr;
        // pinned with the panel: always there, copied in now if it was only reserved ("no slot right
        // now" cannot happen for a pinned tile; should it, it is reported as what it means)
        const int frc = fetch(own, &b);
        if (frc != 0) return frc < 0 ? BLASX_ERR_ARENA_TOO_SMALL : frc;
        if (fill_seq_[b->slot] > 0 && be_.stream_wait_event(d2h, fill_event(b->slot))) return BLASX_ERR_DEVICE;
    }
    BX_TRY(profiled_copy_begin(d2h));
    if (be_.copy_d2h(t.c_host, (size_t)p_->ldc * es, slot_ptr(r.c_slot), (size_t)T_ * es, (size_t)t.m * es, (size_t)t.n, d2h))
        return BLASX_ERR_DEVICE;
    BX_TRY(profiled_copy_end(d2h));
    WriteBack w;            // the caller records the event that covers this copy
    w.slot = r.c_slot;
    ++stats_.copies_d2h;
    stats_.bytes_d2h += (uint64_t)t.m * t.n * es;
    if (p_->results_are_operands) {
        TileRef c;
        c.host = t.c_host;
        c.ld = p_->ldc;
        c.rows = t.m;
        c.cols = t.n;
        w.key = key_of(c);
        w.block = cache_.adopt(w.key, r.c_slot);
        if (!w.block) return BLASX_ERR_DEVICE;
        // a result that later calls may find in the cache as an operand: pad it like a fetched tile (after
        // the launch that wrote it, which is already on the compute stream)
        BX_TRY(zero_padding(r.c_slot, t.m, t.n, STREAM_COMPUTE));
        cache_.acquire(w.block);
    }
    writebacks_.push_back(w);
    task_issued_[r.task] = 1;
    ++stats_.tasks;
    if (t.panel >= 0) {
        PanelState& ps = panels_[t.panel];
        if (--ps.remaining == 0) {
            for (Block* b : ps.blocks) cache_.release(b);
            ps.blocks.clear();
        }
    }
    r.done = true;
    return 0;
}

int Scheduler::start_task(int task_index, Running* r) {
    const Task& t = p_->tasks[task_index];
    if (t.panel >= 0) BX_TRY(ensure_panel(t.panel));
    int slot = -1;
    BX_TRY(take_slot_blocking(&slot));
    *r = Running();
    r->task = task_index;
    r->c_slot = slot;
    if (t.load_c && !late_c_) {
        TileRef c;
        c.host = t.c_host;
        c.ld = p_->ldc;
        c.rows = t.m;
        c.cols = t.n;
        BX_TRY(issue_h2d(c, slot));
    }
    task_started_[task_index] = 1;
    return 0;
}

// Wide mode: start the inbound copy of a task's host C tile into a slot of its own (the
// accumulator slot holds partial sums by then).  Without may_wait nothing is evicted-by-waiting:
// if no slot is free right now the copy is simply started later.
int Scheduler::prefetch_c(Running& r, const Task& t, bool may_wait) {
    if (r.h_slot >= 0) return 0;
    int slot = -1;
    if (may_wait) BX_TRY(take_slot_blocking(&slot));
    else slot = cache_.take_slot();
    if (slot < 0) return 0;
    TileRef c;
    c.host = t.c_host;
    c.ld = p_->ldc;
    c.rows = t.m;
    c.cols = t.n;
    BX_TRY(issue_h2d(c, slot));
    r.h_slot = slot;
    return 0;
}

// Wide mode, a task whose first launch is its last: the host C tile goes straight into the
// task's own slot (nothing has been accumulated there yet).
int Scheduler::load_c_direct(Running& r, const Task& t) {
    if (r.c_direct) return 0;
    TileRef c;
    c.host = t.c_host;
    c.ld = p_->ldc;
    c.rows = t.m;
    c.cols = t.n;
    BX_TRY(issue_h2d(c, r.c_slot));
    r.c_direct = true;
    return 0;
}

// Wide mode: the order in which the running tasks (running_[i] is task i) get their chain of
// `round`.  Queue order, except for the triangular solve (one k-step per round): there the tasks
// solved in this round come first (everyone else's step needs their results), the tasks that
// take their last update in this round -- the launch that also needs the task's own tile of B
// from the host -- come last, and the tasks in between need one tile of A per block row.  The
// copies are prefetched in the same order, so the first update launches of a round wait for a
// handful of tiles instead of a whole block row of B (which is first used a round later).
const std::vector<uint32_t>& Scheduler::round_order(size_t round) {
    const size_t key = p_->results_are_operands || !lag_.empty() ? round : 0;
    int q = 0;                           // an unused entry, else the earliest round
    for (int i = 0; i < kOrders; ++i) {
        if (order_round_[i] == key) return order_[i];
        if (order_round_[q] != SIZE_MAX && (order_round_[i] == SIZE_MAX || order_round_[i] < order_round_[q])) q = i;
    }
    std::vector<uint32_t>& o = order_[q];
    o.clear();
    const size_t n = p_->tasks.size();
    if (!p_->results_are_operands && lag_.empty()) {
        for (size_t i = 0; i < n; ++i) o.push_back((uint32_t)i);
    } else if (!p_->results_are_operands) {
        // staggered panels of tasks of unequal length: chains of one length next to each other, as without the stagger
        auto len = [&](size_t i) -> size_t {
            const long lr = local_round(i, round);
            if (lr < 0) return SIZE_MAX;
            const size_t ns = p_->tasks[i].steps.size();
            const size_t l = std::min(ns, round_begin((size_t)lr + 1)) - std::min(ns, round_begin((size_t)lr));
            return l ? l : SIZE_MAX;
        };
        for (size_t i = 0; i < n; ++i) o.push_back((uint32_t)i);
        std::stable_sort(o.begin(), o.end(), [&](uint32_t x, uint32_t y) { return len(x) < len(y); });
    } else {
        auto cls = [&](size_t i) {
            const long lr = local_round(i, round);      // a trailing column panel is `lag` rounds behind
            if (lr < 0) return 3;
            const size_t ns = p_->tasks[i].steps.size(), r = (size_t)lr;
            return ns == r ? 0 : ns > r + 1 ? 1 : ns == r + 1 ? 2 : 3;
        };
        for (int c = 0; c < 4; ++c)
            for (size_t i = 0; i < n; ++i)
                if (cls(i) == c) o.push_back((uint32_t)i);
    }
    order_round_[q] = key;
    return o;
}

// Wide mode: start the inbound copies of the launches that will be built next, in the order in
// which they will be needed (round by round, in each round's order), up to `prefetch` launches
// ahead.  The host may only run `depth` launches ahead of the device, which is a few milliseconds
// of copies; the copy queue has to be fed further ahead than that or the link idles at every round
// boundary, where a whole new panel of B is needed at once.  Only a hint: build_chain() fetches
// whatever is still missing.
void Scheduler::prefetch_ahead(size_t build_pos) {
    const size_t ntasks = p_->tasks.size();
    const size_t target = build_pos + (size_t)cfg_.prefetch * kMaxStepsPerLaunch;
    // The cursor moves by the tasks of one launch at a time: their tiles are asked for together, sorted so that
    // neighbours in a host matrix follow each other and can share a copy (a launch waits for all of them anyway).
    auto batch_end = [&](size_t pos) {
        const size_t round = pos / ntasks, in_round = pos % ntasks;
        return round * ntasks + std::min(ntasks, (in_round / kMaxStepsPerLaunch + 1) * kMaxStepsPerLaunch);
    };
    struct WantC { Running* r; const Task* t; bool direct; };
    auto c_before = [&](const WantC& x, const WantC& y) {
        const uintptr_t col = (uintptr_t)p_->ldc * p_->esize;
        const uintptr_t rx = (uintptr_t)x.t->c_host % col, ry = (uintptr_t)y.t->c_host % col;
        return rx != ry ? rx < ry : x.t->c_host < y.t->c_host;
    };
    std::vector<const TileRef*> refs;
    std::vector<WantC> want_c;
    if (pf_pos_ < build_pos) pf_pos_ = build_pos;      // the chain about to be built included: its tiles are asked for in sorted order too
    while (pf_pos_ <= target) {
        const size_t round = pf_pos_ / ntasks;
        if (round > pf_last_round_) break;                                // nothing left in any task
        const std::vector<uint32_t>& order = round_order(round);
        const size_t end = batch_end(pf_pos_);
        refs.clear();
        want_c.clear();
        bool beyond = false;
        for (size_t pos = pf_pos_; pos < end; ++pos) {
            const size_t ri = order[pos % ntasks];
            if (ri >= running_.size()) {
                beyond = true;
                break;
            }
            Running& r = running_[ri];
            if (r.task < 0 || r.done) continue;
            const Task& t = p_->tasks[r.task];
            const size_t nsteps = t.steps.size();
            const long lr = local_round((size_t)r.task, round);
            if (lr < 0) continue;
            const size_t s0 = std::min(nsteps, round_begin((size_t)lr)), s1 = std::min(nsteps, round_begin((size_t)lr + 1));
            for (size_t q = s0; q < s1; ++q) {
                // an operand that another task produces is not on the host yet
                if (!t.steps[q].a_is_dep) refs.push_back(&t.steps[q].a);
                if (!t.steps[q].b_is_dep) refs.push_back(&t.steps[q].b);
            }
            // the host tile of C (of B, for a solve) is wanted by the task's last launch of updates; a solve task
            // without updates wants it for its solve, in its first round
            if (t.load_c && ((s0 < nsteps && s1 >= nsteps) || (t.solve && nsteps == 0 && lr == 0))) want_c.push_back(WantC{&r, &t, s0 == 0});
        }
        if (fetch_sorted(refs, true) != 0) break;       // no slot right now: try again after the next launch
        std::sort(want_c.begin(), want_c.end(), c_before);
        bool stalled = false;
        for (const WantC& w : want_c) {
            if (w.direct) {
                if (w.r->first && load_c_direct(*w.r, *w.t) != 0) stalled = true;
            } else if (prefetch_c(*w.r, *w.t, false) != 0 || w.r->h_slot < 0) {
                stalled = true;
            }
            if (stalled) break;
        }
        if (stalled || beyond) break;
        pf_pos_ = end;
    }
    // Host C tiles are wanted by the last launch of each task only, and the last round is the one
    // in which the link is busiest (its operand tiles in, every result tile out).  They are
    // therefore fetched up to a whole round early, into slots that are free anyway: never at
    // the price of evicting an operand tile.
    const size_t c_target = build_pos + ntasks;
    if (pfc_pos_ < build_pos) pfc_pos_ = build_pos;
    while (pfc_pos_ <= c_target) {
        const size_t round = pfc_pos_ / ntasks;
        if (round > pf_last_round_) break;
        const std::vector<uint32_t>& order = round_order(round);
        const size_t end = batch_end(pfc_pos_);
        want_c.clear();
        bool beyond = false;
        for (size_t pos = pfc_pos_; pos < end; ++pos) {
            const size_t ri = order[pos % ntasks];
            if (ri >= running_.size()) {
                beyond = true;
                break;
            }
            Running& r = running_[ri];
            if (r.task < 0 || r.done || r.h_slot >= 0) continue;
            const Task& t = p_->tasks[r.task];
            const size_t nsteps = t.steps.size();
            const long lr = local_round((size_t)r.task, round);
            if (lr < 0) continue;
            const size_t s0 = std::min(nsteps, round_begin((size_t)lr)), s1 = std::min(nsteps, round_begin((size_t)lr + 1));
            if (s0 < nsteps && s1 >= nsteps && s0 > 0 && t.load_c) want_c.push_back(WantC{&r, &t, false});
        }
        std::sort(want_c.begin(), want_c.end(), c_before);
        bool stalled = false;
        for (const WantC& w : want_c) {
            if ((size_t)(cache_.nslots() - cache_.used_slots()) <= pf_reserve_ || prefetch_c(*w.r, *w.t, false) != 0 ||
                w.r->h_slot < 0) {
                stalled = true;
                break;
            }
        }
        if (stalled || beyond) break;
        pfc_pos_ = end;
    }
}

// Grouped schedule: the operand tiles of the chains that the coming round builds, for all running tasks together and
// in fetch_sorted()'s order, into free slots only (a hint: build_chain() fetches whatever is missing).
void Scheduler::prefetch_grouped_round() {
    if (merge_ <= 1) return;
    std::vector<const TileRef*> refs;
    for (const Running& r : running_) {
        if (r.done || r.task < 0) continue;
        const Task& t = p_->tasks[r.task];
        const int nsteps = (int)t.steps.size();
        for (int q = r.next_step; q < std::min(nsteps, r.next_step + kHintChains * kchain_); ++q) {
            const StepSpec& s = t.steps[q];
            if (s.dep >= 0) break;                           // the chain may end at a step that waits for a producer
            if (!s.a_sym && !s.a_mirror) refs.push_back(&s.a);
            if (!s.b_sym && !s.b_mirror) refs.push_back(&s.b);
        }
    }
    // not when slots are scarce: a tile fetched here holds no reader yet, and a later tile of the batch must not push
    // an earlier one out again
    if ((size_t)(cache_.nslots() - cache_.used_slots()) < refs.size() + 2 * running_.size()) return;
    if (fetch_sorted(refs, false) != 0 || !late_c_) return;
    // then the host tiles of C that the coming launches need, block row by block row
    std::vector<Running*> want_c;
    for (Running& r : running_) {
        if (r.done || r.task < 0 || r.h_slot >= 0 || r.c_direct) continue;
        const Task& t = p_->tasks[r.task];
        if (t.load_c && r.next_step + kchain_ >= (int)t.steps.size()) want_c.push_back(&r);
    }
    const uintptr_t col = (uintptr_t)p_->ldc * p_->esize;
    std::sort(want_c.begin(), want_c.end(), [&](const Running* x, const Running* y) {
        const char *cx = p_->tasks[x->task].c_host, *cy = p_->tasks[y->task].c_host;
        const uintptr_t rx = (uintptr_t)cx % col, ry = (uintptr_t)cy % col;
        return rx != ry ? rx < ry : cx < cy;
    });
    for (Running* r : want_c) {
        const Task& t = p_->tasks[r->task];
        if (r->first ? load_c_direct(*r, t) != 0 : (prefetch_c(*r, t, false) != 0 || r->h_slot < 0)) return;
    }
}

// One task per distinct diagonal tile that the solve tasks of a problem invert, in queue order.
std::vector<const Task*> Scheduler::diag_tasks(const Problem& p) const {
    std::vector<const Task*> out;
    std::unordered_set<TileKey, TileKeyHash> seen;
    for (const Task& t : p.tasks)
        if (t.solve && seen.insert(key_of(t.diag, 1 + (int)((t.diag_flags >> 4) & 3u))).second) out.push_back(&t);
    return out;
}

// Wide mode needs an accumulator slot per task plus the operand tiles of two rounds (the round
// being computed and the one being copied in) plus some slots for late C tiles.
bool Scheduler::wide_fits(const Problem& p) {
    std::unordered_set<TileKey, TileKeyHash> uniq;
    size_t max_steps = 0, with_c = 0;
    for (const Task& t : p.tasks) {
        max_steps = std::max(max_steps, t.steps.size());
        with_c += t.load_c ? 1 : 0;
        for (const StepSpec& s : t.steps) {
            uniq.insert(key_of(s.a));
            uniq.insert(key_of(s.b));
        }
    }
    // one launch per task leaves nothing to pipeline, and with barely more than one round the
    // grouped schedule (whose tasks finish one after the other) measures better
    // (the triangular product, whose tasks the wide schedule sorts by length and advances one
    // k-tile per round up to 14 tiles, and the triangular solve, one k-tile per round with its
    // inverses made up front, pay from a third of that: 5 x 5 tiles +10 %, 8 x 8 tiles +40 .. +50 %)
    const size_t least = p.results_are_operands || !p.panels.empty() ? ((size_t)cfg_.wide + 2) / 3
                                                                     : (size_t)cfg_.wide * (size_t)p.steps_per_k;
    if (max_steps <= (size_t)kchain_ || max_steps < least) return false;
    // operand tiles of one full round (the left-over steps make a shorter round of their own)
    const size_t per_round = (uniq.size() * std::min<size_t>(kchain_, max_steps) + max_steps - 1) / max_steps;
    const size_t late_c = with_c ? std::min<size_t>(with_c, (size_t)kMaxStepsPerLaunch * (cfg_.prefetch + cfg_.depth + 2)) : 0;
    pf_reserve_ = per_round + kMaxStepsPerLaunch;
    size_t pinned = 0;      // TRMM: the original tiles of the matrix updated in place stay for the whole call
    for (const Panel& pn : p.panels) pinned += pn.tiles.size();
    // TRSM: diagonal tile, inverse and a scratch tile per block row while the inverses are made up front
    if (p.results_are_operands) pinned += 3 * diag_tasks(p).size();
    return (size_t)cache_.nslots() >= p.tasks.size() + pinned + 2 * per_round + late_c + kMaxStepsPerLaunch;
}

// Next launch of one running task: up to kchain consecutive k-steps (Alg. 1 lines 19-25 for one
// task and one k), operands translated through the cache.  Returns 1 if nothing could be issued
// because a producer task has not been issued yet.
int Scheduler::build_chain(int ri) {
    Running& r = running_[ri];
    const Task& t = p_->tasks[r.task];
    const int nsteps = (int)t.steps.size();
    if (wide_) prefetch_ahead(build_pos_);
    const long lr = wide_ ? local_round((size_t)r.task, round_) : 0;
    if (lr < 0) return 1;                   // a trailing column panel of the solve: not its turn yet
    if (r.next_step >= nsteps && !(r.first && !t.solve)) {
        if (t.solve && !r.solved) return build_solve(ri);
        return 1;
    }
    TileStep st;
    std::memset(&st, 0, sizeof(st));
    Block* held[2 * kMaxChain];
    int nheld = 0, nseg = 0;
    double flops = 0;
    const bool ta = p_->ta, tb = p_->tb;
    // wide mode: up to the end of the current round (the first round may be a short one)
    int chain_limit = kchain_;
    if (wide_) chain_limit = std::max(1, std::min(kchain_, (int)round_begin((size_t)lr + 1) - r.next_step));
    while (nseg < chain_limit && r.next_step + nseg < nsteps) {
        const StepSpec& s = t.steps[r.next_step + nseg];
        if (s.dep >= 0) {
            if (task_final_pack_[s.dep] == 0) break;          // producer's last launch not built yet
            if (pack_is_open(task_final_pack_[s.dep])) BX_TRY(flush_all());
        }
        Block *ba = nullptr, *bb = nullptr;
        const int sym_kind = s.sym_lower ? kDerivedSymLower : kDerivedSymUpper;
        int rc = s.a_sym ? fetch_derived(s.a, sym_kind, &ba) : s.a_mirror ? fetch_derived(s.a, kDerivedTranspose, &ba) : fetch(s.a, &ba);
        if (rc == 0) {
            cache_.acquire(ba);
            rc = s.b_sym ? fetch_derived(s.b, sym_kind, &bb) : s.b_mirror ? fetch_derived(s.b, kDerivedTranspose, &bb) : fetch(s.b, &bb);
            if (rc == 0) cache_.acquire(bb);
            else cache_.release(ba);
        }
        if (rc > 0) return rc;
        if (rc < 0) {
            if (nseg > 0) break;          // issue what fits; the rest follows in the next round
            ++stats_.slot_waits;
            BX_TRY(flush_all());
            if (!inflight_.empty()) retire(true);
            else if (!writebacks_.empty()) poll_writebacks(true);
            else return BLASX_ERR_ARENA_TOO_SMALL;
            poll_writebacks(false);
            continue;
        }
        held[nheld++] = ba;
        held[nheld++] = bb;
        st.seg[nseg].A = slot_ptr(ba->slot);
        st.seg[nseg].B = slot_ptr(bb->slot);
        st.seg[nseg].k = s.k;
        st.seg[nseg].flags = s.seg_flags;
        flops += ((s.seg_flags & (TS_TRI_A | TS_TRI_B)) || t.c_flags ? 1.0 : 2.0) * t.m * t.n * s.k;
        ++nseg;
    }
    if (nseg == 0 && nsteps > 0 && r.next_step < nsteps) return 1;   // blocked on a producer
    // last launch of the task's k loop (a solve task still has its diagonal step to come, which then
    // finds the combined tile alpha * B - sum(A X) in the task's slot)
    const bool last = r.next_step + nseg >= nsteps;
    int acc_slot = -1;          // wide mode: accumulator that the last launch only reads
    st.C = slot_ptr(r.c_slot);
    st.beta = r.first ? t.beta_first : 1.0;
    if (late_c_) {
        // The host C tile is not needed before the task's last launch: earlier launches build
        // alpha * sum(A B) in the accumulator slot, the last one computes
        // alpha * (its products) + beta * C_host + accumulator  into the slot holding C_host.
        if (!last) {
            st.beta = r.first ? 0.0 : 1.0;
        } else if (t.load_c) {
            if (r.first) {
                BX_TRY(load_c_direct(r, t));      // single launch: the tile goes straight into the accumulator slot
            } else {
                BX_TRY(prefetch_c(r, t, true));
                acc_slot = r.c_slot;
                st.D = slot_ptr(acc_slot);
                st.C = slot_ptr(r.h_slot);
                st.beta = t.beta_first;
            }
        }
    }
    st.nseg = (uint16_t)nseg;
    st.lda = st.ldb = st.ldc = (uint16_t)T_;
    st.m = (uint16_t)t.m;
    st.n = (uint16_t)t.n;
    st.flags = (ta ? TS_TRANS_A : 0u) | (tb ? TS_TRANS_B : 0u) | t.c_flags;
    // Every operand tile is zero-padded in its slot: those that came from the host when they were copied, those
    // derived from them by the kernels that made them, the results of a solve when they were adopted as operands.
    if (pad_ok_ && step_is_ragged(st, p_->dtype)) st.flags |= TS_PADDED;
    st.alpha = t.alpha_step;
    OpenPack& op = pack_for(step_mode(st, p_->dtype), ta, tb);
    BX_TRY(add_step(op, ta, tb, st, flops, (uint64_t)nseg));
    for (int q = 0; q < nheld; ++q) {
        op.blocks.push_back(held[q]);
        op.wait_slots.push_back(held[q]->slot);
    }
    op.wait_slots.push_back(r.c_slot);
    if (acc_slot >= 0) {
        // the result now lives in the slot of the host tile; the accumulator is free once this launch is done
        op.wait_slots.push_back(r.h_slot);
        op.free_slots.push_back(acc_slot);
        r.c_slot = r.h_slot;
        r.h_slot = -1;
    }
    r.next_step += nseg;
    r.first = false;
    r.last_pack = op.id;
    if (r.next_step >= nsteps && !t.solve) {
        op.finishing.push_back(ri);
        task_final_pack_[r.task] = op.id;
    }
    return 0;
}

// TRSM: inverse of a diagonal tile of the triangular matrix, cached under the tile's host
// address with a tag.  Small diagonal blocks are inverted directly; block pairs are then merged
// level by level:  inv([L11 0; L21 L22]) = [inv11 0; -inv22 L21 inv11  inv22]  (and the mirror
// image for an upper triangle), each merge being two tile steps of the GEMM kernel.
int Scheduler::get_inverse(const Task& t, Block** out) {
    const int tag = 1 + (int)((t.diag_flags >> 4) & 3u);
    const TileKey key = key_of(t.diag, tag);
    if (!cache_.find(key)) {
        const Task* one = &t;
        BX_TRY(make_inverses(&one, 1));
    }
    bool hit;
    *out = cache_.translate(key, &hit);
    return *out ? 0 : BLASX_ERR_ARENA_TOO_SMALL;
}

// Inverts the diagonal tiles of `count` tasks (those not cached yet) together: one base-block
// launch per tile, then every merge level as one set of launches for all the tiles.  A level of
// one 1024 x 1024 tile is a few small products, far too few to fill the device, and the ten
// levels of a tile run one after the other; the levels of many tiles fill it better and cost
// little more than those of one.
int Scheduler::make_inverses(const Task* const* tasks, size_t count, bool prefetch_after_fetch) {
    struct Job {
        Block *src, *inv;
        int tmp, n;
        uint32_t flags;
    };
    std::vector<Job> jobs;
    auto wait_for_room = [&]() -> int {
        BX_TRY(flush_all());
        if (!inflight_.empty()) retire(true);
        else if (!writebacks_.empty()) poll_writebacks(true);
        else return BLASX_ERR_ARENA_TOO_SMALL;
        return 0;
    };
    for (size_t q = 0; q < count; ++q) {
        const Task& t = *tasks[q];
        const int tag = 1 + (int)((t.diag_flags >> 4) & 3u);
        const TileKey key = key_of(t.diag, tag);
        if (cache_.find(key)) continue;
        Job job{nullptr, nullptr, -1, (int)t.diag.rows, t.diag_flags};
        for (;;) {
            const int rc = fetch(t.diag, &job.src);
            if (rc == 0) break;
            if (rc > 0) return rc;
            BX_TRY(wait_for_room());
        }
        cache_.acquire(job.src);
        for (;;) {
            bool hit;
            job.inv = cache_.translate(key, &hit);
            if (job.inv) break;
            BX_TRY(wait_for_room());
        }
        cache_.acquire(job.inv);
        BX_TRY(take_slot_blocking(&job.tmp));
        jobs.push_back(job);
    }
    if (jobs.empty()) return 0;
    if (prefetch_after_fetch && wide_ && !running_.empty()) {
        build_pos_ = 0;
        prefetch_ahead(0);
    }
    BX_TRY(flush_all());
    const size_t es = p_->esize;
    auto at = [&](int slot, int r, int c) { return slot_ptr(slot) + ((size_t)r + (size_t)c * T_) * es; };
    int max_n = 0;
    for (const Job& job : jobs) {
        // the source tile's inbound copy must have landed, and so must any stale copy still
        // queued into the two slots that are about to be written
        for (int slot : {job.src->slot, job.inv->slot, job.tmp}) {
            if (fill_seq_[slot] > compute_waited_[fill_stream_[slot]]) {
                if (be_.stream_wait_event(STREAM_COMPUTE, fill_event(slot))) return BLASX_ERR_DEVICE;
                compute_waited_[fill_stream_[slot]] = fill_seq_[slot];
            }
        }
        // the inverse is an operand of the solve steps: padded like every operand tile (the kernels below write
        // inside its true extent only)
        BX_TRY(zero_padding(job.inv->slot, job.n, job.n, STREAM_COMPUTE));
        if (be_.launch_trtri_blocks(p_->dtype, slot_ptr(job.src->slot), T_, slot_ptr(job.inv->slot), T_, job.n, kTrtriBlock,
                                    job.flags, STREAM_COMPUTE))
            return BLASX_ERR_DEVICE;
        max_n = std::max(max_n, job.n);
    }
    for (int s = kTrtriBlock; s < max_n; s *= 2) {
        for (int phase = 0; phase < 2; ++phase) {
            for (const Job& job : jobs) {
                const int n = job.n, src = job.src->slot, inv = job.inv->slot, tmp = job.tmp;
                const bool lower = (job.flags & TS_TRI_LOWER) != 0;
                for (int o = 0; o + s < n; o += 2 * s) {
                    const int s2 = std::min(s, n - (o + s));   // order of the second block of the pair
                    TileStep st;
                    std::memset(&st, 0, sizeof(st));
                    st.nseg = 1;
                    st.lda = st.ldb = st.ldc = T_;
                    if (lower) {
                        st.m = s2;
                        st.n = s;
                        if (phase == 0) {       // tmp = L21 * inv11
                            st.C = at(tmp, o + s, o);
                            st.seg[0] = TileSeg{at(src, o + s, o), at(inv, o, o), s, TS_TRI_B | TS_TRI_LOWER};
                            st.alpha = 1.0;
                        } else {                // inv21 = -inv22 * tmp
                            st.C = at(inv, o + s, o);
                            st.seg[0] = TileSeg{at(inv, o + s, o + s), at(tmp, o + s, o), s2, TS_TRI_A | TS_TRI_LOWER};
                            st.alpha = -1.0;
                        }
                    } else {
                        st.m = s;
                        st.n = s2;
                        if (phase == 0) {       // tmp = U12 * inv22
                            st.C = at(tmp, o, o + s);
                            st.seg[0] = TileSeg{at(src, o, o + s), at(inv, o + s, o + s), s2, TS_TRI_B};
                            st.alpha = 1.0;
                        } else {                // inv12 = -inv11 * tmp
                            st.C = at(inv, o, o + s);
                            st.seg[0] = TileSeg{at(inv, o, o), at(tmp, o, o + s), s, TS_TRI_A};
                            st.alpha = -1.0;
                        }
                    }
                    st.beta = 0.0;
                    BX_TRY(add_step(pack_for(step_mode(st, p_->dtype), false, false), false, false, st, 1.0 * st.m * st.n * st.seg[0].k, 0));
                }
            }
            BX_TRY(flush_all());
        }
    }
    // sources, inverses and scratch tiles stay reserved until the last merge has run: a marker
    // record that retires after everything issued so far on the compute stream
    InFlight f;
    f.id = next_pack_id_++;
    f.done_ev = new_event();
    if (be_.event_record(f.done_ev, STREAM_COMPUTE)) return BLASX_ERR_DEVICE;
    for (const Job& job : jobs) {
        f.blocks.push_back(job.src);
        f.blocks.push_back(job.inv);
        f.free_slots.push_back(job.tmp);
    }
    inflight_.push_back(std::move(f));
    return 0;
}

// SYMM: a tile made on the device from a stored tile of the symmetric matrix and cached under the
// stored tile's host address with a tag -- the diagonal tile with both triangles filled in
// (kDerivedSymUpper / kDerivedSymLower: which triangle is stored) or the transpose of an
// off-diagonal tile (kDerivedTranspose).  It is made on the compute stream, so every launch
// issued afterwards sees it.  Return values as fetch().
int Scheduler::fetch_derived(const TileRef& t, int kind, Block** out) {
    const TileKey key = key_of(t, kind);
    bool hit = false;
    if (cache_.find(key)) {
        *out = cache_.translate(key, &hit);
        return 0;
    }
    Block* src = nullptr;
    const int rc = fetch(t, &src);
    if (rc) return rc;
    cache_.acquire(src);
    Block* sym = cache_.translate(key, &hit);
    if (!sym) {
        cache_.release(src);
        return -1;
    }
    // the stored tile must have arrived, and a stale inbound copy into the new slot must be over
    for (int slot : {src->slot, sym->slot}) {
        if (fill_seq_[slot] > compute_waited_[fill_stream_[slot]]) {
            if (be_.stream_wait_event(STREAM_COMPUTE, fill_event(slot))) return BLASX_ERR_DEVICE;
            compute_waited_[fill_stream_[slot]] = fill_seq_[slot];
        }
    }
    // on padded extents where tiles are kept padded: the source's padding is zero, so the new tile's is too
    const int d_rows = pad_ok_ ? round_up_to((int)t.rows, kBM) : (int)t.rows;
    const int d_cols = pad_ok_ ? round_up_to((int)t.cols, kBN) : (int)t.cols;
    const int lrc = kind == kDerivedTranspose
                        ? be_.launch_transpose(p_->dtype, slot_ptr(src->slot), T_, d_rows, d_cols, slot_ptr(sym->slot), T_,
                                               STREAM_COMPUTE)
                        : be_.launch_symmetrize(p_->dtype, slot_ptr(src->slot), T_, slot_ptr(sym->slot), T_, d_rows,
                                                kind == kDerivedSymLower, STREAM_COMPUTE);
    if (lrc) return BLASX_ERR_DEVICE;
    // Both tiles keep a reader until the kernel has run: the stored one because it is read, the
    // new one because a block without readers may be evicted at once and its slot handed to an
    // inbound copy, which is not ordered against work on the compute stream.
    cache_.acquire(sym);
    InFlight f;
    f.done_ev = new_event();
    if (be_.event_record(f.done_ev, STREAM_COMPUTE)) return BLASX_ERR_DEVICE;
    f.blocks.push_back(src);
    f.blocks.push_back(sym);
    inflight_.push_back(std::move(f));
    *out = sym;
    return 0;
}

// TRSM diagonal step: X = inv(op(A_ii)) * W (left) or W * inv(op(A_jj)) (right), written to a
// fresh slot because every output column needs all of W.
int Scheduler::build_solve(int ri) {
    Running& r = running_[ri];
    const Task& t = p_->tasks[r.task];
    if (pack_is_open(r.last_pack)) BX_TRY(flush_all());
    if (late_c_ && r.first) BX_TRY(load_c_direct(r, t));   // no update step came before: the right-hand-side tile has not been fetched yet
    Block* inv = nullptr;
    BX_TRY(get_inverse(t, &inv));
    cache_.acquire(inv);
    int c2 = -1;
    {
        const int rc = take_slot_blocking(&c2);
        if (rc) {
            cache_.release(inv);
            return rc;
        }
    }
    TileStep st;
    std::memset(&st, 0, sizeof(st));
    st.C = slot_ptr(c2);
    st.nseg = 1;
    st.lda = st.ldb = st.ldc = T_;
    st.m = t.m;
    st.n = t.n;
    const uint32_t low = t.diag_flags & TS_TRI_LOWER;
    if (!t.solve_on_right) {
        st.seg[0] = TileSeg{slot_ptr(inv->slot), slot_ptr(r.c_slot), t.m, TS_TRI_A | low};
        st.flags = p_->ta ? TS_TRANS_A : 0u;
    } else {
        st.seg[0] = TileSeg{slot_ptr(r.c_slot), slot_ptr(inv->slot), t.n, TS_TRI_B | low};
        st.flags = p_->tb ? TS_TRANS_B : 0u;
    }
    st.alpha = r.first ? t.beta_first : 1.0;   // a task without update steps still owes the alpha
    st.beta = 0.0;
    // both operands are padded: the inverse when it was made, the right-hand side because its slot was filled by the
    // inbound copy of the task's tile of B (every later launch wrote inside the true extent only)
    if (pad_ok_ && step_is_ragged(st, p_->dtype)) st.flags |= TS_PADDED;
    OpenPack& op = pack_for(step_mode(st, p_->dtype), p_->ta, p_->tb);
    BX_TRY(add_step(op, p_->ta, p_->tb, st, 1.0 * t.m * t.n * st.seg[0].k, 1));
    op.blocks.push_back(inv);
    op.wait_slots.push_back(r.c_slot);
    // the fresh slot may have been evicted a moment ago with an inbound copy for its previous owner
    // still queued: the solve, which writes the slot, is ordered after that copy
    op.wait_slots.push_back(c2);
    op.free_slots.push_back(r.c_slot);
    r.c_slot = c2;
    r.first = false;
    r.solved = true;
    r.last_pack = op.id;
    op.finishing.push_back(ri);
    task_final_pack_[r.task] = op.id;
    return 0;
}

// ---------------------------------------------------------------- main loop --------------

int Scheduler::run(Problem& p) {
    const double t0 = now_s();
    t_wait_ = 0;
    p_ = &p;
    T_ = p.T;
    pad_ok_ = T_ % kBM == 0 && T_ % kBN == 0;
    // tiles per inbound copy: as configured, else as many as make 32 MiB (2 .. 8): beyond that a copy gains nothing
    // more from the pause it saves and only delays its first tile
    merge_ = cfg_.merge > 0 ? std::min(cfg_.merge, (int)kMaxMerge)
                            : (int)std::max<size_t>(2, std::min<size_t>(kMaxMerge, ((size_t)32 << 20) / ((size_t)T_ * T_ * p.esize)));
    const size_t ntasks = p.tasks.size();
    next_task_ = 0;
    rs_.clear();
    rs_prio_.clear();
    rs_dirty_ = true;
    running_.clear();
    task_started_.assign(ntasks, 0);
    task_issued_.assign(ntasks, 0);
    task_final_pack_.assign(ntasks, 0);
    panels_.assign(p.panels.size(), PanelState());
    for (size_t q = 0; q < p.panels.size(); ++q) panels_[q].remaining = p.panels[q].ntasks;
    int rc = 0;
    err_ = 0;
    pack_cut_ = (kMaxStepsPerLaunch / 8) * 8;
    held_.stream = -1;
    if (cfg_.profile >= 2) {
        base_ev_ = new_event();
        if (base_ev_ < 0 || be_.event_record(base_ev_, STREAM_COMPUTE)) rc = BLASX_ERR_DEVICE;
    }
    // Wide mode: every task of the call runs at once and all advance k-chunk by k-chunk (an
    // outer-product order).  A launch then shares its operand tiles with many others, so the
    // device has enough products per tile copied from the first launches on, instead of starving
    // while the first few output tiles wait for whole rows of A and columns of B; and result
    // tiles leave during the whole last round instead of in bursts.  The price is an
    // accumulator slot per output tile, so it is used only when the cache has that room.
    // Chain length (k-tiles per launch) unless the caller fixed it:
    //   wide: 8 (fewer, longer launches; fewer rounds); 6 for 12 .. 15 k-tiles and 4 for 9 .. 11, where
    //     8 would leave two rounds only: the device then waits for eight k-tiles of operands before
    //     its first launch and the results leave in two bursts that the outbound link cannot absorb;
    //   grouped: 4 (shorter pipeline stages for the link-bound sizes);
    //   triangular solve, wide: 1 (right-looking: step k of every task below block row k needs the
    //     results of block row k, which are solved in the same round);
    //   triangular product: 1 up to 14 x 14 tiles in either schedule, 3 for 15 and 16, then as the
    //     others: it has half the products per byte, so the link bounds it up to twice the order, and
    //     its tasks differ in length: one k-tile per launch lets every launch start as soon as its own
    //     few tiles have landed and lets the short tasks' results leave from the first round on.
    size_t longest = 0;
    for (const Task& t : p.tasks) longest = std::max(longest, t.steps.size());
    const bool tri_product = !p.panels.empty();
    int wide_chain = kMaxChain, grouped_chain = 4;
    if (tri_product) {
        wide_chain = longest <= 14 ? 1 : longest <= 16 ? 3 : kMaxChain;
        if (longest <= 14) grouped_chain = 1;
    } else if (longest >= 12 && longest < 16) {
        wide_chain = 6;
    } else if (longest >= 9 && longest < 12) {
        wide_chain = 4;      // 11 k-tiles (the least for the wide schedule by default): rounds of 3 + 4 + 4
    }
    kchain_ = p.results_are_operands ? 1 : cfg_.kchain ? cfg_.kchain : wide_chain;
    wide_ = cfg_.wide > 0 && (int)ntasks > cfg_.group && wide_fits(p);
    // Grouped schedule with room for every tile of the call and a second slot per running task (the link-bound sizes):
    // the host tile of C is fetched for a task's last launch only, as in the wide schedule, and launches are two
    // k-tiles long.  What is left to do when the last inbound tile has landed is then one short launch and its results
    // going out, instead of the whole k loop of the last group.
    late_c_ = wide_;
    if (!wide_ && cfg_.late_c && !p.results_are_operands && p.panels.empty()) {
        std::unordered_set<TileKey, TileKeyHash> uniq;
        for (const Task& t : p.tasks)
            for (const StepSpec& s : t.steps) {
                uniq.insert(key_of(s.a));
                uniq.insert(key_of(s.b));
            }
        late_c_ = (size_t)cache_.nslots() >= uniq.size() + 2 * (size_t)cfg_.group * (cfg_.depth + 2) + kMaxStepsPerLaunch;
        if (late_c_) grouped_chain = std::min(grouped_chain, 2);
        // Such a call is bound by the link, and the queue order decides what is left to do when the last tile has
        // landed.  Block row by block row, every row after the first asks for the same few new tiles (its tiles of
        // the left operand and of C) per unit of work, so copies and launches stay in step to the end; super-block
        // shells end in a corner whose operands are all cached, and its products queue up behind the link.
        if (late_c_ && cfg_.row_order)
            std::stable_sort(p.tasks.begin(), p.tasks.end(),
                             [](const Task& a, const Task& b) { return a.ti != b.ti ? a.ti < b.ti : a.tj < b.tj; });
    }
    if (!wide_) kchain_ = cfg_.kchain ? cfg_.kchain : grouped_chain;
    // Length of the first round.  The last round is the one in which every result tile leaves and
    // every late C tile arrives: a short one cannot hide that traffic.  So the left-over steps are
    // taken first, not last; and when there are none the first full round is split into one of two
    // steps and one of the rest, which starts the device a few milliseconds earlier and still
    // leaves a full last round.  With only two rounds the remainder stays where it was.
    first_chain_ = second_chain_ = kchain_;
    if (wide_ && !p.results_are_operands && kchain_ > 2) {
        size_t max_steps = 0;
        for (const Task& t : p.tasks) max_steps = std::max(max_steps, t.steps.size());
        if (cfg_.ramp > 0) {
            first_chain_ = std::min(cfg_.ramp, kchain_);
        } else if (max_steps >= 2 * (size_t)kchain_) {
            if (max_steps % kchain_) {
                first_chain_ = (int)(max_steps % kchain_);
            } else {
                first_chain_ = 2;
                second_chain_ = kchain_ - 2;
            }
        }
    }
    const int group = wide_ ? (int)ntasks : cfg_.group;
    // A launch lasts as long as its longest chain.  Where the tasks differ in length (TRMM: task
    // (i, j) has as many k-steps as block row i has tiles in the triangle), tasks of equal length
    // are therefore put next to each other: the chains of a round then come out sorted and every
    // launch holds chains of (nearly) one length.  Shortest first: the first launches need the
    // fewest tiles, so the device starts early, and the short tasks' results leave during the
    // call instead of queueing behind its end.
    if (wide_ && !p.results_are_operands)
        std::stable_sort(p.tasks.begin(), p.tasks.end(),
                         [](const Task& a, const Task& b) { return a.steps.size() < b.steps.size(); });
    round_ = 0;
    for (size_t& key : order_round_) key = SIZE_MAX;
    pf_pos_ = pfc_pos_ = 0;
    pf_last_round_ = 0;
    lag_.clear();
    if (wide_) {
        size_t max_steps = 0;
        for (const Task& t : p.tasks) max_steps = std::max(max_steps, t.steps.size());
        while (round_begin(pf_last_round_ + 1) < max_steps) ++pf_last_round_;
        // Wide triangular solve and triangular product: the right-hand sides are cut into `stagger_panels` panels of
        // block columns (block rows when the triangular matrix is on the right), which do not depend on each other,
        // and panel q runs q * stagger_lag rounds behind panel 0.  All panels in step would finish their last block
        // rows, where a round is a few launches long, in one burst that the outbound link needs several times as long
        // to carry, and would start with nothing to compute while the first block row of every panel comes in;
        // staggered, the burst of one panel leaves under the product-rich early rounds of the next.  It pays when
        // the device, not the link, bounds the call (else the smaller launches of two panels only cost): unless a
        // lag is given, the panels are staggered by half of the rounds (the product with fewer than five rounds: by
        // one) when the call's flop at 70 (single precision: 140) TFLOP/s take longer than its inbound bytes at
        // 55 GB/s.  The product's chains of a round are then sorted by length across the panels (round_order()).
        const size_t nrounds = pf_last_round_ + 1;
        if ((p.results_are_operands || !p.panels.empty()) && cfg_.stagger_panels > 1 && cfg_.stagger_lag >= 0 && nrounds >= 3) {
            auto panel_of = [](const Task& t) { return t.panel >= 0 ? t.panel : t.solve_on_right ? t.ti : t.tj; };
            int nb = 0;
            for (const Task& t : p.tasks) nb = std::max(nb, panel_of(t) + 1);
            const int panels = std::min(cfg_.stagger_panels, nb);
            size_t lag = std::min<size_t>((size_t)cfg_.stagger_lag, nrounds);
            if (cfg_.stagger_lag == 0) {
                std::unordered_set<TileKey, TileKeyHash> uniq;
                double bytes_in = 0;
                for (const Task& t : p.tasks) {
                    if (t.load_c) bytes_in += (double)t.m * t.n * p.esize;
                    for (const StepSpec& st : t.steps)
                        if (!st.a_is_dep && uniq.insert(key_of(st.a)).second) bytes_in += (double)st.a.rows * st.a.cols * p.esize;
                    for (const StepSpec& st : t.steps)
                        if (!st.b_is_dep && uniq.insert(key_of(st.b)).second) bytes_in += (double)st.b.rows * st.b.cols * p.esize;
                }
                const bool device_bound = p.flops / (p.dtype == 0 ? 70e12 : 140e12) > bytes_in / 55e9;
                lag = !device_bound ? 0 : p.results_are_operands ? (nrounds + 1) / 2 : nrounds >= 5 ? nrounds / 2 : 1;
            }
            if (panels > 1 && lag > 0) {
                lag_.resize(ntasks);
                size_t lag_max = 0;
                for (size_t i = 0; i < ntasks; ++i) {
                    const Task& t = p.tasks[i];
                    lag_[i] = (uint32_t)((size_t)(panel_of(t) * panels / nb) * lag);
                    lag_max = std::max<size_t>(lag_max, lag_[i]);
                }
                pf_last_round_ += lag_max;
            }
        }
    }
    // Tiles kept from earlier calls: whatever overlaps the matrix this call writes is stale from
    // now on (and must not collide with result tiles adopted under the same host address).
    cache_.forget_evictions();
    if (cache_.blocks()) invalidate_region(p.c_host, p.ldc, p.c_rows, p.c_cols, (int)p.esize);

    // Wide triangular solve: every diagonal tile is fetched and inverted before anything else.
    // Made on demand, the inverse of block row k stands between rounds k - 1 and k: its diagonal
    // tile would be requested behind all the copies already queued, and its ten merge levels keep
    // the device nearly idle for half a millisecond per round.
    bool inverses_first = wide_ && p.results_are_operands;
    if (rc == 0 && wide_ && !p.panels.empty()) rc = reserve_all_panels();

    for (; rc == 0;) {
        retire(false);
        poll_writebacks(false);
        // keep `group` tasks running: top-priority tasks of the reservation station
        if (!wide_) refill_rs();
        size_t active = 0;
        for (const Running& r : running_) active += r.done ? 0 : 1;
        while ((int)active < group) {
            int task = -1;
            if (wide_) {                     // everything starts at once, in queue order
                if (next_task_ < ntasks) task = (int)next_task_++;
            } else {
                task = pick_from_rs();
                if (task < 0 && active == 0) {
                    // nothing runs and the station only holds tasks of panels not entered yet (those of
                    // the open panels are further down the queue): enter one more rather than stop
                    force_open_ = true;
                    task = pick_from_rs();
                    force_open_ = false;
                }
            }
            if (task < 0) break;
            Running r;
            rc = start_task(task, &r);
            if (rc) break;
            bool placed = false;
            for (Running& slot : running_)
                if (slot.done) {
                    slot = r;
                    placed = true;
                    break;
                }
            if (!placed) running_.push_back(r);
            ++active;
            if (!wide_) refill_rs();
        }
        if (rc) break;
        if (inverses_first) {
            // (once every task has its slot: the copies of the first rounds are queued behind the diagonal tiles
            // before the host turns to the many small launches that make the inverses)
            inverses_first = false;
            const std::vector<const Task*> diag = diag_tasks(p);
            rc = make_inverses(diag.data(), diag.size(), true);
            if (rc) break;
        }
        if (active == 0) {
            if (rs_.empty() && next_task_ >= ntasks) break;
            rc = BLASX_ERR_DEVICE;   // tasks remain but none can start: broken dependency order
            break;
        }
        // one round: the next chain of every running task (step k of all tasks before k+1)
        bool progressed = false;
        if (wide_) {
            const std::vector<uint32_t> order = round_order(round_);     // a copy: prefetching asks for other rounds
            for (size_t pos = 0; pos < order.size() && !rc; ++pos) {
                const size_t ri = order[pos];
                if (ri >= running_.size() || running_[ri].done) continue;
                build_pos_ = round_ * ntasks + pos;
                // The results of the very last launch leave with nothing left to hide them: the last sixteen tasks of
                // the last round go out as four launches of four, so that twelve of their tiles leave under a kernel.
                pack_cut_ = cfg_.tail_cut > 0 && round_ == pf_last_round_ && order.size() - pos <= (size_t)kMaxStepsPerLaunch
                                ? std::min(cfg_.tail_cut, (kMaxStepsPerLaunch / 8) * 8)
                                : (kMaxStepsPerLaunch / 8) * 8;
                const int brc = build_chain((int)ri);
                if (brc == 0) progressed = true;
                else if (brc != 1) rc = brc;
            }
        } else {
            prefetch_grouped_round();
            for (size_t ri = 0; ri < running_.size() && !rc; ++ri) {
                if (running_[ri].done) continue;
                const int brc = build_chain((int)ri);
                if (brc == 0) progressed = true;
                else if (brc != 1) rc = brc;
            }
        }
        if (rc) break;
        rc = flush_all();
        if (rc) break;
        ++round_;
        if (!progressed) {
            // every running task waits for a producer that is itself not running: cannot happen
            // with a dependency-ordered queue, but never spin
            rc = BLASX_ERR_DEVICE;
            break;
        }
        while ((int)inflight_.size() > cfg_.depth) retire(true);
    }

    // drain: wait for everything that was issued, even after an error
    {
        if (rc == 0) rc = flush_all();
        if (rc == 0 && err_) rc = err_;
        held_.stream = -1;
        while (!inflight_.empty()) retire(true);
        poll_writebacks(true);
        const double tw = now_s();
        if (be_.sync_all() && rc == 0) rc = BLASX_ERR_DEVICE;
        t_wait_ += now_s() - tw;
    }
    dissect_time();
    for (PanelState& ps : panels_) {
        for (Block* b : ps.blocks) cache_.release(b);
        ps.blocks.clear();
    }
    for (Running& r : running_) {
        if (!r.done && r.c_slot >= 0) cache_.give_slot(r.c_slot);
        if (!r.done && r.h_slot >= 0) cache_.give_slot(r.h_slot);
    }
    running_.clear();
    pending_wb_.clear();
    // What stays cached must equal the host matrices as this call leaves them: operand tiles do,
    // TRSM result tiles do (they were written back from these very slots); original tiles of a
    // matrix updated in place (TRMM) do not.  After an error nothing is trusted.
    if (rc != 0) invalidate_all();
    else if (!p.results_are_operands && cache_.blocks()) invalidate_region(p.c_host, p.ldc, p.c_rows, p.c_cols, (int)p.esize);

    stats_.hits += cache_.hits;
    stats_.misses += cache_.misses;
    stats_.evictions += cache_.evictions;
    stats_.refetches += cache_.refetches;
    stats_.peak_slots = std::max<uint64_t>(stats_.peak_slots, cache_.peak_used);
    cache_.hits = cache_.misses = cache_.evictions = cache_.refetches = 0;
    const double dt = now_s() - t0;
    stats_.t_total_s += dt;
    stats_.t_wait_s += t_wait_;
    stats_.t_issue_s += dt - t_wait_;
    p_ = nullptr;
    return rc;
}

}  // namespace blasx
