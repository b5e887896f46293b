// Host-side bookkeeping of the chunk pool: which fixed-size slot of the pinned pool
// holds which chunk id (the storage manager's "CPU memory addresses of the stored KV
// cache", paper section 4), a lowest-free-first slot allocator, pin counts
// (section 7, Table 3), in-flight counts (the reference counter of section 5.3
// "Zero-Copy Operations": a slot is not released while a transfer still uses it) and
// the order of last use that optional eviction goes by.
// Plain C++, no HIP: usable in an index-only context.
#pragma once

#include <cstdint>
#include <vector>

namespace lmc {

// FNV-1a 64 over a byte string.
inline uint64_t fnv1a64(const uint8_t *p, size_t n, uint64_t h = 0xcbf29ce484222325ull) {
    for (size_t i = 0; i < n; i++) {
        h ^= p[i];
        h *= 0x100000001b3ull;
    }
    return h;
}

// id of a chunk given the id of the chunk before it: FNV-1a over LE64(prev) then the
// tokens as LE32.  Chaining makes an id stand for the whole prefix up to the chunk's end.
inline uint64_t chunk_id(uint64_t prev, const int32_t *tok, int32_t n) {
    uint8_t b[8];
    for (int k = 0; k < 8; k++) b[k] = uint8_t(prev >> (8 * k));
    uint64_t h = fnv1a64(b, 8);
    for (int32_t t = 0; t < n; t++) {
        uint32_t v = uint32_t(tok[t]);
        uint8_t w[4] = {uint8_t(v), uint8_t(v >> 8), uint8_t(v >> 16), uint8_t(v >> 24)};
        h = fnv1a64(w, 4, h);
    }
    return h;
}

// Set of free slot numbers with "take the lowest" in O(levels): a tree of 64-bit words,
// bit set = subtree has a free slot.
class FreeSlots {
public:
    void reset(int64_t n) {
        n_ = n;
        levels_.clear();
        int64_t m = n;
        do {
            m = (m + 63) / 64;
            levels_.emplace_back(size_t(m), 0ull);
        } while (m > 1);
        for (int64_t i = 0; i < n; i++) release(i);
        free_ = n;
    }
    int64_t free_count() const { return free_; }
    // lowest free slot, marked used; -1 when none
    int64_t take_lowest() {
        if (free_ == 0) return -1;
        int64_t idx = 0;
        for (int lv = int(levels_.size()) - 1; lv >= 0; lv--)
            idx = idx * 64 + __builtin_ctzll(levels_[size_t(lv)][size_t(idx)]);
        clear_bit(idx);
        free_--;
        return idx;
    }
    void release(int64_t slot) {
        int64_t idx = slot;
        for (size_t lv = 0; lv < levels_.size(); lv++) {
            uint64_t &w = levels_[lv][size_t(idx / 64)];
            bool was_zero = (w == 0);
            w |= 1ull << (idx % 64);
            idx /= 64;
            if (!was_zero) break;
        }
        free_++;
    }

private:
    void clear_bit(int64_t slot) {
        int64_t idx = slot;
        for (size_t lv = 0; lv < levels_.size(); lv++) {
            uint64_t &w = levels_[lv][size_t(idx / 64)];
            w &= ~(1ull << (idx % 64));
            if (w != 0) break;
            idx /= 64;
        }
    }
    int64_t n_ = 0, free_ = 0;
    std::vector<std::vector<uint64_t>> levels_;
};

struct SlotMeta {
    uint64_t id = 0;
    int32_t pins = 0;
    int32_t inflight = 0;      // enqueued transfers that read or write this slot
    int32_t refs = 0;          // readers that use the slot's bytes in place (lmc_chunk_acquire)
    uint64_t ready_ticket = 0; // the store whose D2H fills this slot (0 = already filled)
    void *ready_event = nullptr;  // while ready_ticket != 0: the event (a hipEvent_t of that store) after
                                  // which this slot's bytes are in the pool; null = the store's last event
    uint64_t use_call = 0;     // number of the last store / retrieve call that used the chunk
    int64_t older = -1, newer = -1;  // neighbours in the order of last use
    bool used = false;
};

// chunk id -> slot: open addressing, linear probing, deletion by backward shift.
class ChunkIndex {
public:
    void reset(int64_t n_slots) {
        meta_.assign(size_t(n_slots), SlotMeta());
        size_t cap = 16;
        while (cap < size_t(n_slots) * 2) cap <<= 1;
        table_.assign(cap, -1);
        mask_ = cap - 1;
        free_.reset(n_slots);
        used_ = 0;
        oldest_ = newest_ = -1;
    }
    int64_t n_slots() const { return int64_t(meta_.size()); }
    int64_t used() const { return used_; }
    SlotMeta &meta(int64_t slot) { return meta_[size_t(slot)]; }

    int64_t find(uint64_t id) const {
        for (size_t i = home(id);; i = (i + 1) & mask_) {
            int64_t s = table_[i];
            if (s < 0) return -1;
            if (meta_[size_t(s)].id == id) return s;
        }
    }
    // lowest free slot bound to id (id must be absent); -1 when the pool is full
    int64_t insert(uint64_t id) {
        int64_t s = free_.take_lowest();
        if (s < 0) return -1;
        SlotMeta &m = meta_[size_t(s)];
        m = SlotMeta();
        m.id = id;
        m.used = true;
        size_t i = home(id);
        while (table_[i] >= 0) i = (i + 1) & mask_;
        table_[i] = s;
        used_++;
        link_newest(s);
        return s;
    }
    void erase(uint64_t id) {
        size_t i = home(id);
        for (;; i = (i + 1) & mask_) {
            int64_t s = table_[i];
            if (s < 0) return;
            if (meta_[size_t(s)].id == id) break;
        }
        int64_t slot = table_[i];
        // close the gap so that every remaining key stays reachable from its home
        size_t hole = i;
        for (size_t j = (i + 1) & mask_; table_[j] >= 0; j = (j + 1) & mask_) {
            size_t h = home(meta_[size_t(table_[j])].id);
            bool between = (hole <= j) ? (hole < h && h <= j) : (hole < h || h <= j);
            if (!between) {
                table_[hole] = table_[j];
                hole = j;
            }
        }
        table_[hole] = -1;
        unlink(slot);
        meta_[size_t(slot)].used = false;
        free_.release(slot);
        used_--;
    }

    // The chunk in `slot` has just been used: it becomes the newest.
    void touch(int64_t slot) {
        if (newest_ == slot) return;
        unlink(slot);
        link_newest(slot);
    }
    // The least recently used chunk that may go: not pinned, no transfer in flight, no
    // reader holding it, not used by call number `call` (a call never evicts what it uses itself); -1 if none.
    int64_t victim(uint64_t call) const {
        for (int64_t s = oldest_; s >= 0; s = meta_[size_t(s)].newer) {
            const SlotMeta &m = meta_[size_t(s)];
            if (m.pins == 0 && m.inflight == 0 && m.refs == 0 && m.use_call != call) return s;
        }
        return -1;
    }
    int64_t oldest() const { return oldest_; }

private:
    void link_newest(int64_t s) {
        SlotMeta &m = meta_[size_t(s)];
        m.older = newest_;
        m.newer = -1;
        if (newest_ >= 0) meta_[size_t(newest_)].newer = s;
        newest_ = s;
        if (oldest_ < 0) oldest_ = s;
    }
    void unlink(int64_t s) {
        SlotMeta &m = meta_[size_t(s)];
        if (m.older >= 0) meta_[size_t(m.older)].newer = m.newer; else oldest_ = m.newer;
        if (m.newer >= 0) meta_[size_t(m.newer)].older = m.older; else newest_ = m.older;
        m.older = m.newer = -1;
    }
    size_t home(uint64_t id) const { return size_t((id * 0x9E3779B97F4A7C15ull) >> 17) & mask_; }
    std::vector<SlotMeta> meta_;
    std::vector<int64_t> table_;
    size_t mask_ = 0;
    FreeSlots free_;
    int64_t used_ = 0;
    int64_t oldest_ = -1, newest_ = -1;  // ends of the order of last use
};

}  // namespace lmc
