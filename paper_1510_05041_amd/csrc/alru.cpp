#include "alru.h"

namespace blasx {

Alru::Alru(int nslots) : nslots_(nslots) {
    free_.reserve(nslots);
    for (int s = nslots - 1; s >= 0; --s) free_.push_back(s);   // slot 0 is handed out first
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

void Alru::give_slot(int slot) { free_.push_back(slot); }

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

std::vector<int> Alru::lru_order() const {
    std::vector<int> out;
    for (Block* b = head_; b; b = b->next) out.push_back(b->slot);
    return out;
}

}  // namespace blasx
