// Dynamic offloading (paper section 5.3) on top of the library's own C ABI: the pages in
// the window are duplicated to the pinned pool with lmc_store, one chunk per block, in
// batches; a query that needs free pages is granted them only once they are duplicated.
#include <hip/hip_runtime.h>

#include <deque>
#include <new>
#include <vector>

#include "../../include/lmc.h"
#include "lmc_window.hpp"

namespace {
constexpr int kBatchBuffers = 4;
struct Flight {
    uint64_t ticket;
    int64_t pages;
    int buffer;
};
}  // namespace

struct lmc_window {
    lmc_ctx_t *ctx = nullptr;
    lmc::OffloadWindow win{1};
    int64_t block_size = 0, max_batch = 0;
    int64_t *host_slots[kBatchBuffers] = {};
    int64_t *dev_slots[kBatchBuffers] = {};
    bool busy[kBatchBuffers] = {};
    std::deque<Flight> flights;    // stores in flight, oldest first
};

namespace {
// Move the current pointer over the stores that have finished (in order).
lmc_status_t poll(lmc_window *w, bool block) {
    while (!w->flights.empty()) {
        Flight &f = w->flights.front();
        lmc_status_t rc = LMC_OK;
        if (f.ticket != 0) rc = block ? lmc_wait(w->ctx, f.ticket) : lmc_test(w->ctx, f.ticket);
        if (rc == LMC_ERR_BUSY) return LMC_OK;
        if (rc != LMC_OK && rc != LMC_ERR_BADSLOT) return rc;
        w->win.completed(f.pages);
        w->busy[f.buffer] = false;
        w->flights.pop_front();
    }
    return LMC_OK;
}
}  // namespace

extern "C" {

lmc_status_t lmc_window_create(lmc_ctx_t *ctx, int64_t window_pages, int64_t max_batch_pages,
                               lmc_window_t **out) {
    if (!ctx || !out || window_pages < 1 || max_batch_pages < 1) return LMC_ERR_INVAL;
    *out = nullptr;
    // a page of the free region is one block over all layers: the context's chunk must be
    // exactly one block
    const int64_t bs = lmc_block_size(ctx);
    if (bs != lmc_chunk_tokens(ctx)) return LMC_ERR_INVAL;
    lmc_window *w = new (std::nothrow) lmc_window();
    if (!w) return LMC_ERR_NOMEM;
    w->ctx = ctx;
    w->win = lmc::OffloadWindow(window_pages);
    w->block_size = bs;
    w->max_batch = max_batch_pages;
    const size_t bytes = size_t(max_batch_pages) * size_t(bs) * 8;
    for (int b = 0; b < kBatchBuffers; b++) {
        if (hipHostMalloc(reinterpret_cast<void **>(&w->host_slots[b]), bytes, hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&w->dev_slots[b]), bytes) != hipSuccess) {
            lmc_window_destroy(w);
            return LMC_ERR_NOMEM;
        }
    }
    *out = w;
    return LMC_OK;
}

lmc_status_t lmc_window_destroy(lmc_window_t *w) {
    if (!w) return LMC_ERR_INVAL;
    (void)poll(w, true);
    for (int b = 0; b < kBatchBuffers; b++) {
        if (w->dev_slots[b]) (void)hipFree(w->dev_slots[b]);
        if (w->host_slots[b]) (void)hipHostFree(w->host_slots[b]);
    }
    delete w;
    return LMC_OK;
}

lmc_status_t lmc_window_release(lmc_window_t *w, const int64_t *blocks, const uint64_t *chunk_ids,
                                int64_t n) {
    if (!w || n < 0 || (n > 0 && (!blocks || !chunk_ids))) return LMC_ERR_INVAL;
    for (int64_t i = 0; i < n; i++) w->win.release(lmc::FreePage{blocks[i], chunk_ids[i]});
    return LMC_OK;
}

lmc_status_t lmc_window_offload(lmc_window_t *w, void *const *kv_layers, void *stream,
                                int64_t *n_issued_out) {
    if (!w || !kv_layers) return LMC_ERR_INVAL;
    lmc_status_t rc = poll(w, false);
    if (rc != LMC_OK) return rc;
    int64_t issued = 0;
    for (;;) {
        int b = -1;
        for (int i = 0; i < kBatchBuffers; i++)
            if (!w->busy[i]) b = i;
        if (b < 0) break;                       // every batch buffer is in flight: come back later
        std::vector<lmc::FreePage> pages;
        w->win.take_scheduled(w->max_batch, &pages);
        if (pages.empty()) break;
        const int64_t bs = w->block_size;
        std::vector<uint64_t> ids(pages.size());
        for (size_t i = 0; i < pages.size(); i++) {
            ids[i] = pages[i].id;
            for (int64_t o = 0; o < bs; o++) w->host_slots[b][int64_t(i) * bs + o] = pages[i].block * bs + o;
        }
        if (hipMemcpyAsync(w->dev_slots[b], w->host_slots[b], pages.size() * size_t(bs) * 8,
                           hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)) != hipSuccess)
            return LMC_ERR_HIP;
        uint64_t t = 0;
        rc = lmc_store(w->ctx, kv_layers, w->dev_slots[b], ids.data(), int64_t(ids.size()), stream, &t);
        // a full pool means these pages cannot be duplicated; they still leave the window,
        // and their content is simply lost when the engine reuses them
        if (rc != LMC_OK && rc != LMC_ERR_NOMEM) return rc;
        w->busy[b] = true;
        w->flights.push_back(Flight{t, int64_t(pages.size()), b});
        issued += int64_t(pages.size());
    }
    if (n_issued_out) *n_issued_out = issued;
    return LMC_OK;
}

lmc_status_t lmc_window_acquire(lmc_window_t *w, int64_t n, int64_t *blocks_out, int32_t block) {
    if (!w || n < 1 || !blocks_out) return LMC_ERR_INVAL;
    lmc_status_t rc = poll(w, false);
    if (rc != LMC_OK) return rc;
    std::vector<int64_t> got;
    int r = w->win.acquire(n, &got);
    if (r == 1 && block) {
        // wait for the stores in flight; what is still only scheduled needs lmc_window_offload
        if ((rc = poll(w, true)) != LMC_OK) return rc;
        r = w->win.acquire(n, &got);
    }
    if (r == 2) return LMC_ERR_NOMEM;
    if (r == 1) return LMC_ERR_BUSY;
    for (int64_t i = 0; i < n; i++) blocks_out[i] = got[size_t(i)];
    return LMC_OK;
}

lmc_status_t lmc_window_get(lmc_window_t *w, int64_t *start, int64_t *current, int64_t *end,
                            int64_t *tail, int32_t *state) {
    if (!w) return LMC_ERR_INVAL;
    lmc_status_t rc = poll(w, false);
    if (rc != LMC_OK) return rc;
    if (start) *start = w->win.start();
    if (current) *current = w->win.current();
    if (end) *end = w->win.end();
    if (tail) *tail = w->win.tail();
    if (state) *state = w->win.state();
    return LMC_OK;
}

}  // extern "C"
