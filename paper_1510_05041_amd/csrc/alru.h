// Tile cache in HBM: the L1 level of the paper's hierarchy (Section IV.B) with the ALRU
// replacement of Alg. 2 -- a hash map from the host address of a tile to the block that
// holds it, an LRU list, and a reader count per block so that a block still in use by
// asynchronous work is never discarded.  Storage is a fixed set of equal tile slots carved
// from one pre-allocated arena (Section IV.E: no per-tile device allocation); because all
// tiles have the same size the paper's first-fit heap degenerates to a free list.
//
// Readings of Alg. 2 taken here: a hit moves the block to the front (otherwise the list
// would be FIFO, not LRU); Dequeue examines every block including the first and also
// removes the hash-map entry; a new block starts with zero readers and the caller acquires
// it at once; when every block has readers the caller must retire work and retry.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <unordered_map>
#include <unordered_set>
#include <vector>

namespace blasx {

struct TileKey {
    const void* host;   // host address of the tile's first element
    int64_t ld;         // host leading dimension (elements)
    int32_t rows, cols; // stored extent of the tile
    int32_t esize;      // element size in bytes
    int32_t tag;        // 0 = the tile itself; other values name data derived from it
    // Does this tile share an element with the column-major region (base, ld, rows, cols, esize)?
    // Exact when both have the same leading dimension and element size (two views of one parent
    // matrix); otherwise decided on the address intervals, which can only err towards "yes".
    bool overlaps(const void* base, int64_t ld, int64_t rows, int64_t cols, int esize) const;
    bool operator==(const TileKey& o) const {
        return host == o.host && ld == o.ld && rows == o.rows && cols == o.cols && esize == o.esize && tag == o.tag;
    }
};

struct TileKeyHash {
    size_t operator()(const TileKey& k) const {
        uint64_t h = reinterpret_cast<uintptr_t>(k.host) * 0x9E3779B97F4A7C15ull;
        h ^= (uint64_t)k.tag * 0xC2B2AE3D27D4EB4Full + ((uint64_t)k.rows << 32) + (uint64_t)k.cols;
        h ^= h >> 29;
        return (size_t)(h * 0xBF58476D1CE4E5B9ull);
    }
};

struct Block {
    TileKey key;
    int slot = -1;
    int readers = 0;
    bool pending = false;    // the slot is reserved but the tile's inbound copy has not been started yet
    Block* prev = nullptr;   // towards the front (most recently used)
    Block* next = nullptr;   // towards the end (least recently used)
};

class Alru {
public:
    explicit Alru(int nslots);
    ~Alru();
    Alru(const Alru&) = delete;
    Alru& operator=(const Alru&) = delete;

    int nslots() const { return nslots_; }
    int used_slots() const { return nslots_ - (int)free_.size(); }

    // HashMap lookup only: no reordering, no counters (used for priorities, Eq. 2).
    Block* find(const TileKey& key) const;
    // Alg. 2 Translate.  *hit tells whether the tile was already cached; on a miss the
    // returned block has a slot but no data yet.  nullptr: no free slot and nothing evictable.
    Block* translate(const TileKey& key, bool* hit);
    void acquire(Block* b) { ++b->readers; }
    void release(Block* b);

    // Raw slots for output accumulators: they count against the same capacity but are not in
    // the map (a written C tile is never served from the cache: the paper's ephemeral M state).
    int  take_slot();            // -1: nothing free and nothing evictable
    void give_slot(int slot);
    // Turn a raw slot that now holds valid data of `key` into a cached block (front of the list).
    Block* adopt(const TileKey& key, int slot);
    // Forget a cached tile (its host copy is about to change).  Returns false if it has readers.
    bool drop(const TileKey& key);

    // Forget every cached tile (derived ones included) that shares an element with the column-major
    // host region (base, ld, rows, cols, esize); blocks with readers are kept and counted in *busy.
    // Returns the number of blocks dropped.
    size_t invalidate_region(const void* base, int64_t ld, int64_t rows, int64_t cols, int esize, size_t* busy = nullptr);
    // Forget everything without readers.
    size_t invalidate_all(size_t* busy = nullptr);
    // Statistics of misses on evicted tiles are per call: forget which tiles were evicted.
    void forget_evictions() { evicted_.clear(); }
    size_t blocks() const { return map_.size(); }

    // Front-to-back list of slots, for tests.
    std::vector<int> lru_order() const;

    uint64_t hits = 0, misses = 0, evictions = 0, refetches = 0, peak_used = 0;

private:
    int  evict_one();            // Alg. 2 Dequeue: slot of the discarded block, or -1
    void unlink(Block* b);
    void push_front(Block* b);
    void note_used();

    int nslots_;
    std::vector<int> free_;
    std::unordered_map<TileKey, Block*, TileKeyHash> map_;
    std::unordered_set<TileKey, TileKeyHash> evicted_;
    Block* head_ = nullptr;
    Block* tail_ = nullptr;
};

}  // namespace blasx
