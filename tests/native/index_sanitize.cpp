// Host-only driver for csrc/lmc_index.hpp, built with -fsanitize=address,undefined by
// tests/test_host_sanitizers.py: random insert / find / erase sequences on ChunkIndex
// against std::map, lowest-free-first against a std::set, the order of last use and
// the choice of a victim against a std::list, and the chained chunk id against a
// byte-wise reference.  Prints "ok" and exits 0 when everything agrees.
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <list>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "../../paper_2510_09665_amd/csrc/lmc_index.hpp"

#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            std::printf("FAILED %s at line %d\n", #c, __LINE__);        \
            return 1;                                                   \
        }                                                               \
    } while (0)

int main() {
    std::mt19937_64 rng(42);
    for (int64_t n_slots : {1, 2, 63, 64, 65, 4096, 4097, 70000}) {
        lmc::ChunkIndex idx;
        idx.reset(n_slots);
        std::map<uint64_t, int64_t> model;
        std::set<int64_t> free_slots;
        for (int64_t i = 0; i < n_slots; i++) free_slots.insert(i);
        const int steps = n_slots > 10000 ? 300000 : 60000;
        // ids drawn from a small range so that hits, re-inserts and erases all happen,
        // and from a clustered range so that probe sequences collide
        const uint64_t id_range = uint64_t(n_slots) * 3 + 5;
        for (int s = 0; s < steps; s++) {
            uint64_t id = (rng() % id_range) * 0x10000ull;
            int op = int(rng() % 3);
            auto it = model.find(id);
            if (op == 0) {
                CHECK(idx.find(id) == (it == model.end() ? -1 : it->second));
            } else if (op == 1) {
                if (it != model.end()) continue;
                int64_t got = idx.insert(id);
                if (free_slots.empty()) {
                    CHECK(got == -1);
                } else {
                    CHECK(got == *free_slots.begin());
                    free_slots.erase(free_slots.begin());
                    model[id] = got;
                    CHECK(idx.meta(got).used && idx.meta(got).id == id && idx.meta(got).pins == 0);
                }
            } else {
                idx.erase(id);
                if (it != model.end()) {
                    free_slots.insert(it->second);
                    model.erase(it);
                }
            }
            CHECK(idx.used() == int64_t(model.size()));
        }
        for (auto &kv : model) CHECK(idx.find(kv.first) == kv.second);
    }
    // order of last use: insert and touch put a chunk at the newest end, erase removes
    // it; the victim is the oldest that is not pinned, not in flight, not of the call
    for (int64_t n_slots : {1, 3, 64, 500}) {
        lmc::ChunkIndex idx;
        idx.reset(n_slots);
        std::list<uint64_t> order;                       // oldest first
        for (int s = 0; s < 40000; s++) {
            uint64_t id = rng() % uint64_t(n_slots * 2 + 1);
            int op = int(rng() % 6);
            int64_t slot = idx.find(id);
            if (op == 0 && slot < 0) {
                if (idx.insert(id) >= 0) order.push_back(id);
            } else if (op == 1 && slot >= 0) {
                idx.erase(id);
                order.remove(id);
            } else if (op == 2 && slot >= 0) {
                idx.touch(slot);
                order.remove(id);
                order.push_back(id);
            } else if (op == 3 && slot >= 0) {
                idx.meta(slot).pins = int32_t(rng() % 2);
                idx.meta(slot).inflight = int32_t(rng() % 2);
                idx.meta(slot).refs = int32_t(rng() % 3 == 0);
                idx.meta(slot).use_call = rng() % 3;
            } else if (op >= 4) {
                const uint64_t call = rng() % 3;
                uint64_t want = ~0ull;
                for (uint64_t o : order) {
                    const lmc::SlotMeta &m = idx.meta(idx.find(o));
                    if (m.pins == 0 && m.inflight == 0 && m.refs == 0 && m.use_call != call) {
                        want = o;
                        break;
                    }
                }
                const int64_t v = idx.victim(call);
                CHECK((v < 0) == (want == ~0ull));
                if (v >= 0) CHECK(idx.meta(v).id == want);
            }
            CHECK(idx.used() == int64_t(order.size()));
            CHECK((idx.oldest() < 0) == order.empty());
            if (!order.empty()) CHECK(idx.meta(idx.oldest()).id == order.front());
        }
        // walk the whole list once: same ids in the same order
        int64_t sl = idx.oldest();
        for (uint64_t o : order) {
            CHECK(sl >= 0 && idx.meta(sl).id == o);
            sl = idx.meta(sl).newer;
        }
        CHECK(sl == -1);
    }
    // chained id == FNV-1a over the concatenated little-endian message
    std::vector<int32_t> tok(300);
    for (auto &t : tok) t = int32_t(rng());
    for (int n : {1, 16, 256}) {
        uint64_t prev = rng();
        std::vector<uint8_t> msg;
        for (int k = 0; k < 8; k++) msg.push_back(uint8_t(prev >> (8 * k)));
        for (int t = 0; t < n; t++)
            for (int k = 0; k < 4; k++) msg.push_back(uint8_t(uint32_t(tok[size_t(t)]) >> (8 * k)));
        CHECK(lmc::chunk_id(prev, tok.data(), n) == lmc::fnv1a64(msg.data(), msg.size()));
    }
    CHECK(lmc::fnv1a64(reinterpret_cast<const uint8_t *>("foobar"), 6) == 0x85944171f73967e8ull);
    std::printf("ok\n");
    return 0;
}
