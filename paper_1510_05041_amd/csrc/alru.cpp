#include "alru.h"

#include <algorithm>
#include <functional>

namespace blasx {

bool TileKey::overlaps(const void* base, int64_t ld_r, int64_t rows_r, int64_t cols_r, int esize_r) const {
    if (rows <= 0 || cols <= 0 || rows_r <= 0 || cols_r <= 0) return false;
    const char* t0 = static_cast<const char*>(host);
    const char* t1 = t0 + ((int64_t)(cols - 1) * ld + rows) * esize;
    const char* r0 = static_cast<const char*>(base);
    const char* r1 = r0 + ((cols_r - 1) * ld_r + rows_r) * esize_r;
    if (t1 <= r0 || r1 <= t0) return false;
    const int64_t d = t0 - r0;
    if (ld != ld_r || esize != esize_r || d % esize != 0 || rows > ld || rows_r > ld) return true;
    // position of the tile's first element on the region's column grid (floor division)
    const int64_t e = d / esize;
    int64_t c0 = e / ld;
    int64_t q0 = e - c0 * ld;
    if (q0 < 0) {
        q0 += ld;
        --c0;
    }
    auto rect_hits = [&](int64_t row_lo, int64_t row_hi, int64_t col_lo, int64_t col_hi) {
        return row_lo < rows_r && row_hi > 0 && col_lo < cols_r && col_hi > 0 && row_lo < row_hi;
    };
    // rows [q0, q0 + rows) of columns [c0, c0 + cols); a tile that crosses the bottom of the grid
    // continues at the top of the next column
    if (q0 + rows <= ld) return rect_hits(q0, q0 + rows, c0, c0 + cols);
    return rect_hits(q0, ld, c0, c0 + cols) || rect_hits(0, q0 + rows - ld, c0 + 1, c0 + 1 + cols);
}

Alru::Alru(int nslots) : nslots_(nslots) {
    // A min-heap: the lowest free slot is handed out first, so slots taken one after the other are neighbours in
    // the arena whenever a run of them is free (tiles copied in together can then share a strided copy).
    free_.reserve(nslots);
    for (int s = 0; s < nslots; ++s) free_.push_back(s);        // ascending order is a valid min-heap
}

Alru::~Alru() {
    for (auto& kv : map_) delete kv.second;
}

void Alru::unlink(Block* b) {
    if (b->prev) b->prev->next = b->next; else head_ = b->next;
    if (b->next) b->next->prev = b->prev; else tail_ = b->prev;
    b->prev = b->next = nullptr;
}

void Alru::push_front(Block* b) {
    b->prev = nullptr;
    b->next = head_;
    if (head_) head_->prev = b;
    head_ = b;
    if (!tail_) tail_ = b;
}

void Alru::note_used() {
    const uint64_t u = (uint64_t)used_slots();
    if (u > peak_used) peak_used = u;
}

Block* Alru::find(const TileKey& key) const {
    auto it = map_.find(key);
    return it == map_.end() ? nullptr : it->second;
}

// Alg. 2 Dequeue: walk from the least recently used end towards the front and discard the
// first block nobody is reading.
int Alru::evict_one() {
    for (Block* b = tail_; b; b = b->prev) {
        if (b->readers == 0) {
            const int slot = b->slot;
            unlink(b);
            map_.erase(b->key);
            evicted_.insert(b->key);
            delete b;
            ++evictions;
            return slot;
        }
    }
    return -1;
}

int Alru::take_slot() {
    int slot;
    if (!free_.empty()) {
        std::pop_heap(free_.begin(), free_.end(), std::greater<int>());
        slot = free_.back();
        free_.pop_back();
    } else {
        slot = evict_one();
        if (slot >= 0) {            // evict_one does not touch the free list: account for the reuse
            note_used();
            return slot;
        }
        return -1;
    }
    note_used();
    return slot;
}

void Alru::give_slot(int slot) {
    free_.push_back(slot);
    std::push_heap(free_.begin(), free_.end(), std::greater<int>());
}

// Alg. 2 Translate (+ Enqueue on a miss).
Block* Alru::translate(const TileKey& key, bool* hit) {
    if (Block* b = find(key)) {
        *hit = true;
        ++hits;
        if (b != head_) {
            unlink(b);
            push_front(b);
        }
        return b;
    }
    *hit = false;
    const int slot = take_slot();
    if (slot < 0) return nullptr;
    ++misses;
    if (evicted_.count(key)) ++refetches;
    Block* b = new Block();
    b->key = key;
    b->slot = slot;
    b->readers = 0;
    map_.emplace(key, b);
    push_front(b);
    return b;
}

void Alru::release(Block* b) {
    if (b->readers > 0) --b->readers;
}

Block* Alru::adopt(const TileKey& key, int slot) {
    if (Block* old = find(key)) {     // replace a stale copy
        if (old->readers == 0) {
            unlink(old);
            map_.erase(key);
            give_slot(old->slot);
            delete old;
        } else {
            return nullptr;
        }
    }
    Block* b = new Block();
    b->key = key;
    b->slot = slot;
    map_.emplace(key, b);
    push_front(b);
    return b;
}

bool Alru::drop(const TileKey& key) {
    Block* b = find(key);
    if (!b) return true;
    if (b->readers > 0) return false;
    unlink(b);
    map_.erase(key);
    give_slot(b->slot);
    delete b;
    return true;
}

size_t Alru::invalidate_region(const void* base, int64_t ld, int64_t rows, int64_t cols, int esize, size_t* busy) {
    std::vector<Block*> hit;
    for (auto& kv : map_)
        if (kv.first.overlaps(base, ld, rows, cols, esize)) hit.push_back(kv.second);
    size_t dropped = 0;
    for (Block* b : hit) {
        if (b->readers > 0) {
            if (busy) ++*busy;
            continue;
        }
        unlink(b);
        map_.erase(b->key);
        give_slot(b->slot);
        delete b;
        ++dropped;
    }
    return dropped;
}

size_t Alru::invalidate_all(size_t* busy) {
    std::vector<Block*> all;
    for (auto& kv : map_) all.push_back(kv.second);
    size_t dropped = 0;
    for (Block* b : all) {
        if (b->readers > 0) {
            if (busy) ++*busy;
            continue;
        }
        unlink(b);
        map_.erase(b->key);
        give_slot(b->slot);
        delete b;
        ++dropped;
    }
    evicted_.clear();
    return dropped;
}

std::vector<int> Alru::lru_order() const {
    std::vector<int> out;
    for (Block* b = head_; b; b = b->next) out.push_back(b->slot);
    return out;
}

}  // namespace blasx
