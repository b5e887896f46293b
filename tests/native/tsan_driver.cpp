// Thread-sanitizer driver for the library's host side: several threads use one index-only
// context (LMC_DEVICE_NONE, eviction on) at once through the C ABI, among them readers
// that hold counts on chunks and a directory tier whose writer threads read the pool in
// place (its two directories are the program's arguments).  Built and run by
// tests/test_host_tsan.py together with a thread-sanitized build of the library's host code.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/lmc.h"

int main(int argc, char **argv) {
    if (argc != 3) return 2;
    lmc_config_t cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.geom.num_layers = 2; cfg.geom.num_planes = 2; cfg.geom.num_heads = 2; cfg.geom.head_dim = 8;
    cfg.geom.elem_bytes = 2; cfg.geom.block_size = 4; cfg.geom.num_blocks = 64; cfg.geom.chunk_tokens = 16;
    cfg.geom.head_stride = 16; cfg.geom.token_stride = 32; cfg.geom.block_stride = 128;
    cfg.geom.plane_stride = 64 * 128;
    cfg.num_staging = 2; cfg.staging_chunks = 1; cfg.device = LMC_DEVICE_NONE;
    cfg.flags = LMC_FLAG_EVICT_LRU;
    lmc_ctx_t *ctx = nullptr;
    const int64_t chunk = 2 * 2 * 16 * 2 * 8 * 2;
    cfg.host_pool_bytes = 64 * chunk;
    if (lmc_create(&cfg, &ctx) != LMC_OK || lmc_chunk_bytes(ctx) != chunk) return 2;
    lmc_tier_t *tier = nullptr;
    const char *dirs[2] = {argv[1], argv[2]};
    if (lmc_tier_open(ctx, dirs, 2, 3, &tier) != LMC_OK) return 2;
    std::atomic<int> bad{0};
    auto worker = [&](int tid) {
        const size_t n_bytes = static_cast<size_t>(chunk);
        std::vector<uint8_t> buf(n_bytes, static_cast<uint8_t>(tid));
        std::vector<uint8_t> out(n_bytes);
        for (int i = 0; i < 4000; i++) {
            uint64_t id = uint64_t((i * 7 + tid * 13) % 90);
            switch (i % 8) {
                case 0: (void)lmc_put_host(ctx, &id, 1, buf.data()); break;
                case 1: { int64_t n; if (lmc_lookup(ctx, &id, 1, &n) != LMC_OK) bad++; break; }
                case 2: if (lmc_pin(ctx, &id, 1) == LMC_OK && lmc_unpin(ctx, &id, 1) != LMC_OK) bad++; break;
                case 3: (void)lmc_clear(ctx, &id, 1); break;
                case 4: {
                    lmc_status_t rc = lmc_get_host(ctx, id, out.data());
                    // a chunk is always one writer's bytes, never a mixture
                    if (rc == LMC_OK) for (size_t k = 1; k < out.size(); k += 97) if (out[k] != out[0]) bad++;
                    break;
                }
                case 5: {
                    // a counted reader sees one writer's bytes for as long as it holds the count
                    const void *p = nullptr;
                    if (lmc_chunk_acquire(ctx, id, &p) == LMC_OK) {
                        const uint8_t *b = static_cast<const uint8_t *>(p);
                        for (int rep = 0; rep < 3; rep++)
                            for (size_t k = 1; k < n_bytes; k += 61) if (b[k] != b[0]) bad++;
                        if (lmc_chunk_release(ctx, id) != LMC_OK) bad++;
                    }
                    break;
                }
                case 6:
                    if (i % 40 == 6) {
                        lmc_status_t rc = lmc_tier_write(tier, &id, 1);
                        if (rc != LMC_OK && rc != LMC_ERR_MISS) bad++;
                    }
                    break;
                default: { lmc_stats_t st; if (lmc_get_stats(ctx, &st) != LMC_OK || st.pool_slots_used > 64) bad++; }
            }
        }
    };
    std::vector<std::thread> th;
    for (int t = 0; t < 6; t++) th.emplace_back(worker, t);
    for (auto &t : th) t.join();
    if (lmc_tier_wait(tier) != LMC_OK) bad++;
    uint64_t files = 0, bytes = 0, back = 0;
    if (lmc_tier_get_stats(tier, &files, &bytes, &back) != LMC_OK || files == 0 || bytes != files * uint64_t(chunk)) bad++;
    lmc_tier_close(tier);
    lmc_destroy(ctx);
    if (bad.load()) { std::printf("FAILED %d checks\n", bad.load()); return 1; }
    std::printf("ok\n");
    return 0;
}
