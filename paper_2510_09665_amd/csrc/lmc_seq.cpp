// Delayed decode KV storing (paper section 5.1): newly generated tokens are not
// offloaded one by one; a per-sequence accumulator holds them until a whole chunk exists
// and then stores that chunk in one batched operation.  This file is a policy layer on
// top of the library's own C ABI (lmc_hash_chunks_from, lmc_store, lmc_wait): it adds no
// data path of its own.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "../../include/lmc.h"

namespace {
constexpr int kSlotBuffers = 4;  // chunks of this sequence that may be in flight at once
}

struct lmc_seq {
    lmc_ctx_t *ctx = nullptr;
    int32_t chunk_tokens = 0;
    uint64_t last_id = 0;               // id of the last full chunk (or the hash seed)
    bool have_last = false;
    int64_t n_tokens = 0;               // tokens seen so far, prompt included
    std::vector<int32_t> tail_tokens;   // tokens of the chunk that is still filling up
    std::vector<int64_t> tail_slots;
    // slot mappings must live in device memory until the store's gather has run:
    // a small ring of pinned + device buffers, each remembering the ticket that used it
    int64_t *host_slots[kSlotBuffers] = {};
    int64_t *dev_slots[kSlotBuffers] = {};
    uint64_t ticket[kSlotBuffers] = {};
    int next = 0;
};

extern "C" {

lmc_status_t lmc_seq_open(lmc_ctx_t *ctx, const int32_t *prompt_tokens, const int64_t *prompt_slots,
                          int64_t n_prompt, lmc_seq_t **seq_out) {
    if (!ctx || !seq_out || n_prompt < 0 || (n_prompt > 0 && (!prompt_tokens || !prompt_slots)))
        return LMC_ERR_INVAL;
    *seq_out = nullptr;
    lmc_seq *s = new (std::nothrow) lmc_seq();
    if (!s) return LMC_ERR_NOMEM;
    s->ctx = ctx;
    s->chunk_tokens = lmc_chunk_tokens(ctx);
    const int64_t CT = s->chunk_tokens;
    // the prompt's full chunks only advance the id chain: storing them is the prefill's job
    const int64_t n_full = n_prompt / CT;
    if (n_full > 0) {
        std::vector<uint64_t> ids(static_cast<size_t>(n_full));
        int64_t n = 0;
        lmc_status_t rc = lmc_hash_chunks(ctx, prompt_tokens, n_full * CT, ids.data(), &n);
        if (rc != LMC_OK) {
            delete s;
            return rc;
        }
        s->last_id = ids.back();
        s->have_last = true;
    }
    s->tail_tokens.assign(prompt_tokens + n_full * CT, prompt_tokens + n_prompt);
    s->tail_slots.assign(prompt_slots + n_full * CT, prompt_slots + n_prompt);
    s->n_tokens = n_prompt;
    for (int b = 0; b < kSlotBuffers; b++) {
        if (hipHostMalloc(reinterpret_cast<void **>(&s->host_slots[b]), size_t(CT) * 8, hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&s->dev_slots[b]), size_t(CT) * 8) != hipSuccess) {
            lmc_seq_close(s);
            return LMC_ERR_NOMEM;
        }
    }
    *seq_out = s;
    return LMC_OK;
}

lmc_status_t lmc_seq_append(lmc_seq_t *s, const int32_t *tokens, const int64_t *slots, int64_t n,
                            void *const *kv_layers, void *stream, int64_t *n_chunks_offered_out,
                            uint64_t *last_ticket_out) {
    if (!s || n < 0 || (n > 0 && (!tokens || !slots)) || !kv_layers) return LMC_ERR_INVAL;
    const int64_t CT = s->chunk_tokens;
    int64_t offered = 0;
    uint64_t last_ticket = 0;
    lmc_status_t result = LMC_OK;
    for (int64_t i = 0; i < n; i++) {
        s->tail_tokens.push_back(tokens[i]);
        s->tail_slots.push_back(slots[i]);
        s->n_tokens++;
        if (int64_t(s->tail_tokens.size()) < CT) continue;
        // a chunk is complete: its id continues the chain, its slots go to the device,
        // and the library's store takes it from there (a chunk already present is skipped)
        uint64_t id = 0;
        int64_t one = 0;
        lmc_status_t rc = s->have_last
                              ? lmc_hash_chunks_from(s->ctx, s->last_id, s->tail_tokens.data(), CT, &id, &one)
                              : lmc_hash_chunks(s->ctx, s->tail_tokens.data(), CT, &id, &one);
        if (rc != LMC_OK) return rc;
        const int b = s->next;
        s->next = (s->next + 1) % kSlotBuffers;
        if (s->ticket[b] != 0) {
            rc = lmc_wait(s->ctx, s->ticket[b]);      // the buffer's previous store has gathered
            if (rc == LMC_ERR_BADSLOT) result = rc;  // reported once by the library: pass it on
            else if (rc != LMC_OK) return rc;
            s->ticket[b] = 0;
        }
        std::memcpy(s->host_slots[b], s->tail_slots.data(), size_t(CT) * 8);
        if (hipMemcpyAsync(s->dev_slots[b], s->host_slots[b], size_t(CT) * 8, hipMemcpyHostToDevice,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
            return LMC_ERR_HIP;
        uint64_t t = 0;
        rc = lmc_store(s->ctx, kv_layers, s->dev_slots[b], &id, 1, stream, &t);
        s->last_id = id;
        s->have_last = true;
        s->tail_tokens.clear();
        s->tail_slots.clear();
        if (rc != LMC_OK && rc != LMC_ERR_NOMEM) return rc;
        if (rc == LMC_ERR_NOMEM && result == LMC_OK) result = rc;  // the chain moves on; the chunk is not stored
        s->ticket[b] = t;
        last_ticket = t;
        offered++;
    }
    if (n_chunks_offered_out) *n_chunks_offered_out = offered;
    if (last_ticket_out) *last_ticket_out = last_ticket;
    return result;
}

lmc_status_t lmc_seq_pending_tokens(const lmc_seq_t *s, int64_t *n_out) {
    if (!s || !n_out) return LMC_ERR_INVAL;
    *n_out = int64_t(s->tail_tokens.size());
    return LMC_OK;
}

lmc_status_t lmc_seq_close(lmc_seq_t *s) {
    if (!s) return LMC_ERR_INVAL;
    for (int b = 0; b < kSlotBuffers; b++) {
        if (s->ticket[b] != 0) (void)lmc_wait(s->ctx, s->ticket[b]);
        if (s->dev_slots[b]) (void)hipFree(s->dev_slots[b]);
        if (s->host_slots[b]) (void)hipHostFree(s->host_slots[b]);
    }
    delete s;
    return LMC_OK;
}

}  // extern "C"
