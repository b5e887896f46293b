// Thread-sanitizer driver for the library's host side: several threads use one index-only
// context (LMC_DEVICE_NONE) at once through the C ABI.  Built and run by
// tests/test_host_tsan.py together with a thread-sanitized build of the library's host code.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/lmc.h"

int main() {
    lmc_config_t cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.geom.num_layers = 2; cfg.geom.num_planes = 2; cfg.geom.num_heads = 2; cfg.geom.head_dim = 8;
    cfg.geom.elem_bytes = 2; cfg.geom.block_size = 4; cfg.geom.num_blocks = 64; cfg.geom.chunk_tokens = 16;
    cfg.geom.head_stride = 16; cfg.geom.token_stride = 32; cfg.geom.block_stride = 128;
    cfg.geom.plane_stride = 64 * 128;
    cfg.num_staging = 2; cfg.staging_chunks = 1; cfg.device = LMC_DEVICE_NONE;
    lmc_ctx_t *ctx = nullptr;
    const int64_t chunk = 2 * 2 * 16 * 2 * 8 * 2;
    cfg.host_pool_bytes = 64 * chunk;
    if (lmc_create(&cfg, &ctx) != LMC_OK || lmc_chunk_bytes(ctx) != chunk) return 2;
    std::atomic<int> bad{0};
    auto worker = [&](int tid) {
        const size_t n_bytes = static_cast<size_t>(chunk);
        std::vector<uint8_t> buf(n_bytes, static_cast<uint8_t>(tid));
        std::vector<uint8_t> out(n_bytes);
        for (int i = 0; i < 4000; i++) {
            uint64_t id = uint64_t((i * 7 + tid * 13) % 90);
            switch (i % 6) {
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
                default: { lmc_stats_t st; if (lmc_get_stats(ctx, &st) != LMC_OK || st.pool_slots_used > 64) bad++; }
            }
        }
    };
    std::vector<std::thread> th;
    for (int t = 0; t < 6; t++) th.emplace_back(worker, t);
    for (auto &t : th) t.join();
    lmc_destroy(ctx);
    if (bad.load()) { std::printf("FAILED %d checks\n", bad.load()); return 1; }
    std::printf("ok\n");
    return 0;
}
