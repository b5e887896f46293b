/*
 * lmc.h -- C ABI of liblmc: batched movement of KV cache between an inference
 * engine's paged GPU memory and contiguous fixed-size token chunks in pinned host
 * memory, for AMD MI355X (gfx950).
 *
 * The operations are the ones the paper describes for its KV caching layer:
 *   - section 5.1 "Configurable Chunk Size": pages of many layers are grouped into
 *     chunks (default 256 tokens); on store a kernel copies the scattered pages into
 *     a contiguous streaming GPU buffer that is then moved to CPU memory as one
 *     transfer per chunk; on load the chunk is moved back into the buffer and a
 *     kernel splits it into pages;
 *   - section 4 "Store" / "Retrieve": a token processor decides which tokens are new
 *     (only those are stored) and how many leading tokens of a prompt are already
 *     present (only those are loaded); a storage manager keeps the CPU addresses;
 *   - section 1 (#1) and 5.2: store and load are batched and pipelined so that the
 *     copy kernels overlap the transfers;
 *   - section 7, Table 3: lookup / pin / unpin / clear, here in their local,
 *     single-instance form.
 *
 * Conventions
 *   - Every function returns an lmc_status_t; nothing throws or aborts.  A NULL
 *     pointer where one is required gives LMC_ERR_INVAL.
 *   - "DEVICE" pointers are HIP device addresses on the context's GPU; "HOST" pointers
 *     are ordinary process memory.  The library never takes ownership of a caller's
 *     buffer.  No torch or C++ type crosses this boundary.
 *   - Paged KV memory is described by lmc_kv_geom_t: one allocation per layer, and in
 *     it the run of head_dim*elem_bytes bytes of (plane p, block b, in-block token o,
 *     head h) starts at
 *         kv_layers[l] + p*plane_stride + b*block_stride + o*token_stride + h*head_stride.
 *     kv_layers is a HOST array of num_layers DEVICE pointers; it is read during the
 *     call only.  The pages themselves and the slot mapping must stay alive and
 *     unmodified (store) / unread (retrieve) until lmc_wait returns for the ticket.
 *   - A chunk is chunk_tokens tokens over all layers and planes, laid out
 *     [layer][plane][token][head][dim], dense; lmc_chunk_bytes() bytes.
 *   - A slot mapping is a DEVICE array of int64, one entry per token:
 *     slot = block*block_size + in-block offset.  A negative slot means the token has
 *     no page: store writes zeros for it into the chunk, retrieve writes nothing for
 *     it.  A slot >= num_blocks*block_size is never dereferenced; it is reported as
 *     LMC_ERR_BADSLOT (see lmc_wait and LMC_FLAG_VALIDATE_SLOTS).  Two tokens of one
 *     retrieve call that name the same slot leave that slot's content unspecified.
 *   - A chunk id is a 64-bit value, normally from lmc_hash_chunks.  Equal ids mean
 *     the same chunk.
 *   - One context may be used from several threads; calls are serialised inside.
 */
#ifndef LMC_H
#define LMC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lmc_ctx lmc_ctx_t; /* opaque, owned by the library */
typedef int32_t lmc_status_t;

enum {
    LMC_OK = 0,
    LMC_ERR_INVAL = -1,    /* bad argument or geometry */
    LMC_ERR_NOMEM = -2,    /* host pool full, or an allocation failed */
    LMC_ERR_MISS = -3,     /* a chunk id is not in the pool */
    LMC_ERR_BADSLOT = -4,  /* a slot >= num_blocks*block_size */
    LMC_ERR_HIP = -5,      /* a HIP call failed; lmc_last_hip_error() has its code */
    LMC_ERR_BUSY = -6,     /* chunk pinned or in flight */
    LMC_ERR_NODEVICE = -7, /* data-movement call on an index-only context */
    LMC_ERR_IO = -8        /* a file of a lower tier could not be written or read */
};

#define LMC_MAX_LAYERS 160        /* kv_layers travels as a kernel argument */
#define LMC_STATIC_SCRATCH_BYTES (64ull << 20) /* device memory of lmc_store_static, per GPU */
#define LMC_DEVICE_NONE (-1)      /* index-only context: see lmc_create */

/* lmc_config_t.flags */
#define LMC_FLAG_VALIDATE_SLOTS 1u /* check every slot mapping on the device before any
                                      byte moves; a bad slot then fails the call itself
                                      with LMC_ERR_BADSLOT and nothing is written.  Costs
                                      one small kernel and a host wait per call. */
#define LMC_FLAG_FORCE_SYNC 2u     /* wait for the device after every enqueue step: the
                                      pipeline runs serially.  Same results, for debugging. */
#define LMC_FLAG_POISON_STAGING 4u /* overwrite a staging buffer with 0xA5 as soon as the
                                      pipeline releases it: a reuse that came too early
                                      then shows as corrupt data.  For tests. */
#define LMC_FLAG_DIRECT 16u        /* no staging buffer and no copy engine for any call: the
                                      gather kernel writes, and the scatter kernel reads, the
                                      pinned pool over the host link (64 workgroups, resident
                                      for the length of the transfer).  Same results.
                                      Without the flag only calls of at most 64 MiB go this
                                      way (lmc_tune "direct_store_below" / "..._retrieve_below"). */
#define LMC_FLAG_EVICT_LRU 32u     /* a new chunk that finds the pool full takes the slot of
                                      the least recently used chunk that is not pinned, has
                                      no transfer in flight and is not used by the same
                                      call; within one call's chunks the later position is
                                      the older one (a request loses its tail first, and
                                      what is left still hits as a prefix).  Uses are
                                      lmc_store (new and present chunks), lmc_put_host and
                                      the retrieve calls; lookup, pin, unpin are not.  The
                                      paper names no policy (sections 4.2, 7); without the
                                      flag a full pool gives LMC_ERR_NOMEM. */
#define LMC_FLAG_KEEP_STREAMS 64u   /* leave the library's six streams on the hardware queues
                                      the runtime gave them.  Without the flag lmc_create (pool
                                      and staging buffer of 8 MiB or more) spends some tens of
                                      milliseconds finding out which streams share a queue and
                                      picks, from a few more than it needs, streams such that
                                      the two kernel streams and the first copy stream of each
                                      direction have four different queues: the four streams
                                      of a store and a retrieve running together then never
                                      wait for each other. */
#define LMC_FLAG_TRACE 128u         /* keep a record of every pipeline step (see lmc_trace_read);
                                      also switched by lmc_tune("trace", 0 / 1).  Costs two
                                      event markers per group on the copy streams. */
#define LMC_FLAG_TIMING 8u         /* give every gather / scatter launch a start and a stop
                                      HIP event (kernel begin / end on its own stream);
                                      durations appear in lmc_stats_t. */

/* Geometry of the engine's paged KV memory (section 5: a page is block_size tokens of
 * one layer) and the chunk length (section 5.1).  All strides are in bytes. */
typedef struct {
    int32_t num_layers;   /* 1 .. LMC_MAX_LAYERS */
    int32_t num_planes;   /* 2 = K and V, 1 = a single latent (MLA) */
    int32_t num_heads;
    int32_t head_dim;     /* elements */
    int32_t elem_bytes;   /* 2 = bf16 / fp16, 1 = fp8; payload is opaque bytes */
    int32_t block_size;   /* tokens per page */
    int32_t num_blocks;   /* pages per layer and plane; num_blocks*block_size < 2^31 */
    int32_t chunk_tokens; /* 256 by default in the paper */
    int64_t plane_stride, block_stride, token_stride, head_stride; /* >= 0 */
} lmc_kv_geom_t;
/* Each layer's allocation must cover every run the strides can reach:
 *   (P-1)*plane_stride + (NB-1)*block_stride + (BS-1)*token_stride + (H-1)*head_stride
 *   + head_dim*elem_bytes bytes.
 * The kernels move min(16, largest power of two dividing head_dim*elem_bytes and every
 * stride) bytes per lane; the layer base pointers and staging_dev must be aligned to
 * that, else LMC_ERR_INVAL.  16-byte multiples everywhere give the fast path. */

typedef struct {
    lmc_kv_geom_t geom;
    uint64_t host_pool_bytes; /* pinned pool; holds host_pool_bytes / chunk_bytes chunks */
    int32_t num_staging;      /* staging buffers per direction, >= 2 (double buffering) */
    int32_t staging_chunks;   /* chunks per staging buffer, >= 1: one kernel launch covers
                                 up to this many chunks.  The group at the exposed end of
                                 a pipeline (first of a store, last of a retrieve) is a
                                 single chunk. */
    int32_t device;           /* HIP device ordinal, or LMC_DEVICE_NONE */
    uint32_t flags;           /* LMC_FLAG_* */
    uint64_t hash_seed;       /* "hash before the first chunk" of lmc_hash_chunks */
} lmc_config_t;

typedef struct {
    uint64_t pool_slots_total, pool_slots_used;
    uint64_t chunks_stored;       /* written by lmc_store / lmc_put_host */
    uint64_t chunks_skipped_dup;  /* offered to lmc_store but already present */
    uint64_t chunks_retrieved;
    uint64_t retrieve_misses;     /* calls refused with LMC_ERR_MISS */
    uint64_t alloc_failures;      /* calls that hit LMC_ERR_NOMEM */
    uint64_t chunks_evicted;      /* LMC_FLAG_EVICT_LRU: chunks that gave up their slot */
    uint64_t d2h_guard_switches;  /* times the copies to the host went over to the copy kernel */
    uint64_t d2h_guard_active;    /* 1 while they are with the copy kernel, else 0 */
    uint64_t bytes_gathered, bytes_scattered; /* chunk payload through the kernels */
    uint64_t bytes_d2h, bytes_h2d;            /* chunk payload over the host link */
    uint64_t gather_launches, scatter_launches;
    uint64_t timed_gather_launches, timed_scatter_launches; /* LMC_FLAG_TIMING, completed */
    double gather_ms, scatter_ms;             /* sum of their HIP-event durations */
    double d2h_copy_best_gbps;    /* best rate seen of a runtime copy to the host of 32 MiB or
                                     more (what "d2h_guard" compares with); 0 = none seen */
    double d2h_copy_last_gbps;    /* rate of the latest such copy */
} lmc_stats_t;

/* Create a context (section 4: the storage manager that owns the CPU memory the KV cache
 * is offloaded to; section 5.1: the contiguous streaming GPU buffers between the pages
 * and that memory): allocates the pinned host pool, 2*num_staging device staging
 * buffers of staging_chunks chunks each (one ring per direction), six HIP streams
 * and the index.  With device == LMC_DEVICE_NONE nothing touches HIP: the pool is
 * ordinary host memory and only the host-side calls work (hashing, lookup, put/get,
 * pin/unpin/clear, stats); every call that would move data to or from a GPU returns
 * LMC_ERR_NODEVICE.  There is no CPU implementation of the data path.
 * Errors: LMC_ERR_INVAL (a geometry field out of the ranges given at lmc_kv_geom_t,
 * num_staging < 2, staging_chunks < 1 or more than one launch can cover, pool smaller
 * than one chunk), LMC_ERR_NOMEM (pool or staging cannot be allocated), LMC_ERR_HIP. */
lmc_status_t lmc_create(const lmc_config_t *cfg, lmc_ctx_t **ctx_out);
/* Waits for outstanding work, then frees everything the context owns. */
lmc_status_t lmc_destroy(lmc_ctx_t *ctx);

int64_t lmc_chunk_bytes(const lmc_ctx_t *ctx); /* chunk_tokens*layers*planes*heads*dim*elem */
int32_t lmc_chunk_tokens(const lmc_ctx_t *ctx);
int32_t lmc_block_size(const lmc_ctx_t *ctx);
int64_t lmc_pool_slots(const lmc_ctx_t *ctx);

/* Token processor (section 4): chained 64-bit ids of the full chunks of a token
 * sequence.  id_i = FNV-1a-64( LE64(id_{i-1}) || LE32(tok[i*CT]) .. LE32(tok[i*CT+CT-1]) ),
 * id_{-1} = hash_seed; a tail shorter than chunk_tokens is ignored.  tokens: HOST
 * int32[n_tokens]; ids_out: HOST, room for n_tokens / chunk_tokens values;
 * n_chunks_out: HOST, receives that count. */
lmc_status_t lmc_hash_chunks(const lmc_ctx_t *ctx, const int32_t *tokens, int64_t n_tokens,
                             uint64_t *ids_out, int64_t *n_chunks_out);
/* The same chain continued: prev_id is the id of the chunk just before tokens[0]. */
lmc_status_t lmc_hash_chunks_from(const lmc_ctx_t *ctx, uint64_t prev_id, const int32_t *tokens,
                                  int64_t n_tokens, uint64_t *ids_out, int64_t *n_chunks_out);

/* Prefix match (section 4 "Retrieve"): n_hit_out receives the number of leading ids
 * that are all present.  A later isolated hit does not count.  HOST pointers. */
lmc_status_t lmc_lookup(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n,
                        int64_t *n_hit_out);

/* Store (sections 4 and 5.1).  For each of the n_chunks chunks in order: if its id is
 * present it is skipped (first writer wins); otherwise it takes the lowest free pool
 * slot, is gathered from the pages into a staging buffer and copied to that slot (a
 * call with few new bytes, or any call under LMC_FLAG_DIRECT, is gathered straight into
 * the slot).
 * slot_mapping: DEVICE int64[n_chunks*chunk_tokens].  chunk_ids: HOST.
 * stream_to_wait_on: a hipStream_t (NULL names the null stream): the library's work is
 * ordered after everything enqueued on it so far (the kernels that produced the KV and
 * the slot mapping).
 * The call only enqueues; *ticket_out (HOST, may be NULL) names the work for lmc_wait.
 * A stored chunk is visible to lmc_lookup at once; a retrieve of it is ordered after
 * the store on the device, group by group: the copy of a chunk to the device waits for the
 * copies of the store's group that holds the chunk, not for the whole store, so a retrieve
 * enqueued right behind the store of the same chunks runs beside it (both directions of
 * the link at work).
 * Errors: LMC_ERR_NOMEM when the pool fills: chunks before the failing one are stored
 * and their work is still covered by the ticket.  LMC_ERR_BADSLOT under
 * LMC_FLAG_VALIDATE_SLOTS (nothing stored).  LMC_ERR_NODEVICE.  LMC_ERR_HIP: the call
 * waits for what it had enqueued and takes back every chunk it had admitted (none of
 * them is visible afterwards, their slots are free again; chunks evicted to make room
 * stay evicted); no ticket is issued. */
lmc_status_t lmc_store(lmc_ctx_t *ctx, void *const *kv_layers, const int64_t *slot_mapping,
                       const uint64_t *chunk_ids, int64_t n_chunks, void *stream_to_wait_on,
                       uint64_t *ticket_out);

/* Retrieve (sections 4 and 5.1).  All n_chunks ids must be present, else LMC_ERR_MISS
 * and no page byte is written.  Each chunk is copied from its pool slot into a staging
 * buffer (or, for a small call or under LMC_FLAG_DIRECT, read where it is) and scattered
 * into the pages named by slot_mapping (DEVICE
 * int64[n_chunks*chunk_tokens]); bytes of the pages that no slot names are not
 * touched.  stream_to_signal: a hipStream_t (NULL names the null stream).  The scatter
 * is ordered after everything enqueued on it so far (earlier users of the pages, the
 * producer of the slot mapping), and the stream is made to wait for the last scatter,
 * so work enqueued on it afterwards sees the pages (unless lmc_tune "caller_waits" is 0:
 * then the caller orders its work after lmc_wait itself).  Enqueue only.
 * LMC_ERR_HIP in the middle of the call: what had been enqueued is waited for, no count
 * stays on the chunks, no ticket is issued; the pages named by slot_mapping are then
 * partly written. */
lmc_status_t lmc_retrieve(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n_chunks,
                          const int64_t *slot_mapping, void *const *kv_layers,
                          void *stream_to_signal, uint64_t *ticket_out);

/* Retrieve for many requests in one call.  Request r owns chunks
 * [req_chunk_offsets[r], req_chunk_offsets[r+1]) of chunk_ids and of slot_mapping
 * (HOST int64[n_req+1], starting at 0, non-decreasing).  One missing chunk anywhere
 * gives LMC_ERR_MISS and nothing is written.  Kernel launches span request borders. */
lmc_status_t lmc_retrieve_batch(lmc_ctx_t *ctx, int64_t n_req, const int64_t *req_chunk_offsets,
                                const uint64_t *chunk_ids, const int64_t *slot_mapping,
                                void *const *kv_layers, void *stream_to_signal,
                                uint64_t *ticket_out);

/* Layer-wise retrieve (section 5.2 "Layer-wise pipelining"; start_load_kv / wait_load_kv
 * of section 6, Table 2).  Same contract as lmc_retrieve, but the work is ordered by
 * layer: for layers_per_step layers at a time, the share of every chunk in those layers
 * is copied to the staging buffer (one rectangle copy per run of consecutive pool
 * slots) and scattered, then the next layers follow, so that layer l's pages are
 * complete long before the last layer's.  The consumer orders itself per layer with
 * lmc_wait_layer; unlike lmc_retrieve, no stream is made to wait for the whole call.
 * stream_to_wait_on: the call is ordered after work already on it (old users of the
 * pages, producer of the slot mapping).  layers_per_step >= 1 (values above num_layers
 * mean "all").  Errors as lmc_retrieve, and LMC_ERR_BUSY if one of the chunks belongs
 * to a layer-wise store whose layers have not all been submitted. */
lmc_status_t lmc_retrieve_layerwise(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n_chunks,
                                    const int64_t *slot_mapping, void *const *kv_layers,
                                    int32_t layers_per_step, void *stream_to_wait_on,
                                    uint64_t *ticket_out);

/* Layer-wise store (section 5.2; start_store_kv / wait_store_kv of Table 2): the KV of a
 * forward pass becomes available layer by layer, and each layer is offloaded as soon as
 * it exists.  lmc_store_begin runs the token processor (which chunks are new, where they
 * go; same rules and errors as lmc_store) and returns a ticket; nothing moves yet.  The
 * slot mapping (DEVICE) must stay alive until lmc_wait(ticket) returns.
 * lmc_store_layers then submits layers [first_layer, first_layer + n_layers): they are
 * gathered from kv_layers and copied into the layer's place inside every new chunk's
 * pool slot, ordered after work already on stream_to_wait_on (the kernels that produced
 * those layers).  Layers must be submitted in ascending order without gaps, else
 * LMC_ERR_INVAL; when the last layer has been submitted the ticket behaves like any
 * other.  Until then lmc_wait on it, lmc_get_host and a retrieve of its chunks return
 * LMC_ERR_BUSY, and its chunks cannot be cleared.  LMC_ERR_HIP from lmc_store_layers
 * ends the whole store: its chunks leave the index, the ticket is void. */
lmc_status_t lmc_store_begin(lmc_ctx_t *ctx, const int64_t *slot_mapping, const uint64_t *chunk_ids,
                             int64_t n_chunks, void *stream_to_wait_on, uint64_t *ticket_out);
lmc_status_t lmc_store_layers(lmc_ctx_t *ctx, uint64_t ticket, int32_t first_layer,
                              int32_t n_layers, void *const *kv_layers, void *stream_to_wait_on);

/* Make `stream` (hipStream_t, NULL = null stream) wait, on the device, until layer
 * `layer` of a layer-wise ticket is in place: loaded into its pages (retrieve) or
 * arrived in the pool (store).  The host does not block.  A finished ticket needs no
 * wait and returns LMC_OK.  LMC_ERR_INVAL for a ticket that is not layer-wise or a
 * layer out of range; LMC_ERR_BUSY for a store layer that has not been submitted. */
lmc_status_t lmc_wait_layer(lmc_ctx_t *ctx, uint64_t ticket, int32_t layer, void *stream);

/* wait_store_kv / wait_load_kv of section 6, Table 2 (bulk form; lmc_wait_layer is the
 * per-layer form): block until the work of `ticket` and of every earlier ticket has
 * finished on the device, whichever of the library's streams each of them ended on;
 * ticket 0 means everything enqueued so far.  Returns LMC_ERR_BADSLOT if a
 * kernel since the last lmc_wait met a slot >= num_blocks*block_size (that token was
 * skipped, the rest of the call was carried out), LMC_ERR_HIP on a device error.
 * A layer-wise store that still lacks layers cannot be waited for: LMC_ERR_BUSY if it
 * is the ticket named (or ticket is 0); an older one is left out of the wait. */
lmc_status_t lmc_wait(lmc_ctx_t *ctx, uint64_t ticket);

/* The non-blocking form of the same two connector calls (section 6, Table 2): has the
 * work of `ticket` finished?  LMC_OK: yes; LMC_ERR_BUSY: not yet (or a layer-wise
 * store still lacks layers).  Never blocks, reports no slot errors. */
lmc_status_t lmc_test(lmc_ctx_t *ctx, uint64_t ticket);

/* The two kernels of section 5.1 alone (store: the pages of a chunk are copied into one
 * contiguous GPU buffer; load: the buffer is split into pages again), for unit parity and
 * for measuring them against HBM
 * bandwidth: pages -> n_chunks contiguous chunks at staging_dev (DEVICE,
 * n_chunks*chunk_bytes, 16-byte aligned) and back.  Enqueued on `stream`
 * (hipStream_t, NULL = the null stream); no host wait except under
 * LMC_FLAG_VALIDATE_SLOTS.  A bad slot is reported by the next lmc_wait. */
lmc_status_t lmc_gather(lmc_ctx_t *ctx, void *const *kv_layers, const int64_t *slot_mapping,
                        int64_t n_chunks, void *staging_dev, void *stream);
lmc_status_t lmc_scatter(lmc_ctx_t *ctx, const void *staging_dev, const int64_t *slot_mapping,
                         int64_t n_chunks, void *const *kv_layers, void *stream);

/* For callers that cannot allocate: tight serving loops, harnesses that forbid hipMalloc
 * after start-up, code that may run while another part of the process captures a HIP
 * graph.  The data path of lmc_store (gather the pages of each chunk into a contiguous
 * device buffer, copy the buffer to host memory) with nothing allocated by the call, on
 * the device or through the runtime: the buffer is a static array of
 * LMC_STATIC_SCRATCH_BYTES in the library's device image (each GPU the library is used on
 * holds its own copy until the process ends; its address is looked up when lmc_create
 * first runs on that GPU), the destination is the caller's, and no event or stream is
 * created.  There is no index, pool or ticket on this path: chunk i of the slot mapping
 * (DEVICE int64[n_chunks*chunk_tokens], same rules as lmc_store) arrives at
 * host_dst + i*lmc_chunk_bytes(), byte for byte what lmc_store would have put into the
 * pool.  host_dst: HOST memory from hipHostMalloc (the runtime copies to pageable memory
 * through buffers of its own), n_chunks*chunk_bytes, caller-owned.
 * Everything is enqueued on `stream` (hipStream_t, NULL = the null stream), kernel and copy
 * in turn, one piece of at most LMC_STATIC_SCRATCH_BYTES at a time; the stream's order is
 * what keeps a piece's kernel off the array until the piece before has been copied out.
 * The work is complete when `stream` has passed it (hipStreamSynchronize or an event of
 * the caller's).  Any n_chunks is taken; a chunk larger than the array goes a few layers
 * at a time.  Calls that overlap on one GPU (other streams, other contexts, other
 * threads) share the array and race: one call at a time per GPU.  Every byte of a piece
 * is written by its gather, so nothing of an earlier call shows through.
 * Errors: LMC_ERR_INVAL (NULL argument; one layer of one chunk is larger than
 * LMC_STATIC_SCRATCH_BYTES; host_dst is not pinned host memory; device ordinal of the
 * context >= 64), LMC_ERR_NODEVICE, LMC_ERR_BADSLOT as for lmc_gather, LMC_ERR_HIP (pieces
 * enqueued before the failing call still complete). */
lmc_status_t lmc_store_static(lmc_ctx_t *ctx, void *const *kv_layers, const int64_t *slot_mapping,
                              int64_t n_chunks, void *host_dst, void *stream);

/* Chunks that arrive from, or leave to, host memory without touching the GPU (a lower
 * storage tier, section 5.1 "Parallel Store/load Operations").  lmc_put_host stores n
 * chunks of lmc_chunk_bytes() each, read back to back from host_src, under the same
 * rules as lmc_store (present ids skipped, lowest free slot, LMC_ERR_NOMEM keeps what
 * was stored).  lmc_get_host copies one chunk to host_dst after waiting for a store of
 * it that is still in flight.  lmc_find_slot reports the pool slot of an id. */
lmc_status_t lmc_put_host(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n,
                          const void *host_src);
lmc_status_t lmc_get_host(lmc_ctx_t *ctx, uint64_t chunk_id, void *host_dst);
lmc_status_t lmc_find_slot(lmc_ctx_t *ctx, uint64_t chunk_id, int64_t *slot_out);

/* Delayed decode storing (section 5.1 "Delayed Decode KV Cache Storing"): tokens
 * generated during decoding are not offloaded one at a time; they are held back until a
 * whole chunk exists, which is then stored in one batched operation.  An lmc_seq_t is
 * that accumulator for one sequence; it is a policy layer over lmc_store and is not
 * thread-safe by itself (one sequence, one caller).
 * lmc_seq_open: prompt_tokens / prompt_slots (HOST, n_prompt entries) describe what the
 *   sequence holds already.  The prompt's full chunks only advance the id chain (storing
 *   them is the prefill's lmc_store); its tail shorter than a chunk starts the pending
 *   chunk.  Allocates a few chunk_tokens-sized slot buffers (pinned and device).
 * lmc_seq_append: n more tokens with their slots (HOST).  Every chunk that becomes
 *   complete gets its chained id, its slot mapping is uploaded on `stream`, and it is
 *   handed to lmc_store (ordered after `stream`; a chunk already present is skipped).
 *   n_chunks_offered_out (may be NULL): chunks completed by this call;
 *   last_ticket_out (may be NULL): ticket of the last store, 0 if none.  kv_layers as in
 *   lmc_store.  LMC_ERR_NOMEM: the pool was full for at least one chunk; the chain moves
 *   on regardless.  The caller's slots arrays are copied and need not stay alive.
 * lmc_seq_pending_tokens: tokens held back so far (always < chunk_tokens).
 * lmc_seq_close: waits for the sequence's stores and frees it; pending tokens are
 *   dropped (only full chunks are ever stored). */
typedef struct lmc_seq lmc_seq_t;
lmc_status_t lmc_seq_open(lmc_ctx_t *ctx, const int32_t *prompt_tokens, const int64_t *prompt_slots,
                          int64_t n_prompt, lmc_seq_t **seq_out);
lmc_status_t lmc_seq_append(lmc_seq_t *seq, const int32_t *tokens, const int64_t *slots, int64_t n,
                            void *const *kv_layers, void *stream, int64_t *n_chunks_offered_out,
                            uint64_t *last_ticket_out);
lmc_status_t lmc_seq_pending_tokens(const lmc_seq_t *seq, int64_t *n_out);
lmc_status_t lmc_seq_close(lmc_seq_t *seq);

/* Dynamic offloading (section 5.3): the engine's free pages form a queue and only a
 * window of them is duplicated to CPU memory.  Three pointers walk the queue: start (head
 * of the free region), current (pages before it are offloaded), end (pages before it are
 * scheduled).  A page here is one block over all layers, stored as one chunk, so the
 * context must have chunk_tokens == block_size (else LMC_ERR_INVAL).  One window, one
 * caller at a time.
 * lmc_window_create: window_pages >= 1 is the target of end - start; max_batch_pages
 *   bounds how many pages one lmc_store call duplicates.
 * lmc_window_release: the engine frees n blocks (HOST arrays): they join the tail with the
 *   ids under which their KV is cached; the end pointer follows until the window is full.
 * lmc_window_offload: start duplicating the scheduled pages that have not been started
 *   yet (lmc_store in batches, ordered after `stream`); n_issued_out may be NULL.  Pages
 *   that find the pool full leave the window without a copy.
 * lmc_window_acquire: a query wants n free pages.  LMC_OK: blocks_out[0..n) are the n
 *   head blocks and the end pointer has moved forward by n.  LMC_ERR_BUSY: the request
 *   stalls, nothing is taken: not all n pages are duplicated yet (a request larger than
 *   the window pulls the end pointer to start + n; call lmc_window_offload and try
 *   again).  With block != 0 the call first waits for the duplications in flight.
 *   LMC_ERR_NOMEM: fewer than n free pages exist.
 * lmc_window_get: pointer positions (absolute counts of pages that ever entered the free
 *   region; any may be NULL) and the section's state number: 1 initialization, 2 in
 *   progress, 4 steady (state 3, query arrival, is the move made by a granted acquire). */
typedef struct lmc_window lmc_window_t;
lmc_status_t lmc_window_create(lmc_ctx_t *ctx, int64_t window_pages, int64_t max_batch_pages,
                               lmc_window_t **window_out);
lmc_status_t lmc_window_destroy(lmc_window_t *w);
lmc_status_t lmc_window_release(lmc_window_t *w, const int64_t *blocks, const uint64_t *chunk_ids,
                                int64_t n);
lmc_status_t lmc_window_offload(lmc_window_t *w, void *const *kv_layers, void *stream,
                                int64_t *n_issued_out);
lmc_status_t lmc_window_acquire(lmc_window_t *w, int64_t n, int64_t *blocks_out, int32_t block);
lmc_status_t lmc_window_get(lmc_window_t *w, int64_t *start, int64_t *current, int64_t *end,
                            int64_t *tail, int32_t *state);

/* Local forms of the controller verbs of section 7, Table 3.  HOST pointers.
 * pin: every id must be present (else LMC_ERR_MISS, nothing pinned); adds one pin each.
 * unpin: every id present (else LMC_ERR_MISS) and pinned often enough (else
 *        LMC_ERR_INVAL); on error nothing changes.
 * clear: removes the ids that are present and frees their slots; absent ids are
 *        ignored; if one is pinned or still in flight the call fails with LMC_ERR_BUSY
 *        and removes nothing. */
lmc_status_t lmc_pin(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n);
lmc_status_t lmc_unpin(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n);
lmc_status_t lmc_clear(lmc_ctx_t *ctx, const uint64_t *chunk_ids, int64_t n);

/* The reference counter of section 5.3 "Zero-Copy Operations": a reader that sends a
 * stored chunk somewhere else (a lower tier, a peer) does not copy it first.
 * lmc_chunk_acquire waits until the chunk's bytes are in the pool (LMC_ERR_BUSY if they
 * belong to a layer-wise store that has not been submitted completely, LMC_ERR_MISS if
 * the chunk is absent), raises the chunk's counter and returns the address of its
 * chunk_bytes bytes in the pinned pool (HOST, read-only, valid until the matching
 * release).  While the counter is above zero the chunk keeps its slot: lmc_clear
 * answers LMC_ERR_BUSY and eviction passes it over.  Several readers each hold their own
 * count.  lmc_chunk_release lowers it: LMC_ERR_MISS if absent, LMC_ERR_INVAL if zero. */
lmc_status_t lmc_chunk_acquire(lmc_ctx_t *ctx, uint64_t chunk_id, const void **host_ptr_out);
lmc_status_t lmc_chunk_release(lmc_ctx_t *ctx, uint64_t chunk_id);

/* A lower tier made of directories, one file per chunk ("local disk and remote object
 * storage" of section 5.3 stand behind mount points here).  lmc_tier_write sends each
 * chunk to EVERY directory at once: one count on the chunk per destination
 * (lmc_chunk_acquire), no copy of the data, writer threads that read the pinned pool in
 * place, one release per finished file.  It returns as soon as the work is queued;
 * all-or-nothing: if one id is absent (LMC_ERR_MISS) or not yet complete
 * (LMC_ERR_BUSY) nothing is queued.  A file appears under its final name
 * (<dir>/<16 hex digits of the id>.kv) only when it is complete.
 * lmc_tier_wait blocks until everything queued has been written and returns LMC_ERR_IO
 * if a file failed since the last wait (errno through lmc_tier_errno); the chunks'
 * counts are given back either way.
 * lmc_tier_lookup: the number of leading ids whose file exists in directory dir.
 * lmc_tier_read brings chunks back from directory dir into the pool: ids already
 * present are skipped, new ones are admitted like lmc_put_host (LMC_ERR_NOMEM when the
 * pool is full and nothing can be evicted; LMC_ERR_MISS if a file is absent,
 * LMC_ERR_IO if it is short or unreadable); ids before the failing one stay.  This
 * direction goes through one bounce buffer.
 * Close the tier (waits for queued writes) before destroying the context.  Calls on
 * one tier may come from several threads.  dirs: HOST strings, copied. */
typedef struct lmc_tier lmc_tier_t;
lmc_status_t lmc_tier_open(lmc_ctx_t *ctx, const char *const *dirs, int32_t n_dirs,
                           int32_t n_threads, lmc_tier_t **tier_out);
lmc_status_t lmc_tier_close(lmc_tier_t *tier);
lmc_status_t lmc_tier_write(lmc_tier_t *tier, const uint64_t *chunk_ids, int64_t n);
lmc_status_t lmc_tier_wait(lmc_tier_t *tier);
lmc_status_t lmc_tier_lookup(lmc_tier_t *tier, int32_t dir, const uint64_t *chunk_ids, int64_t n,
                             int64_t *n_hit_out);
lmc_status_t lmc_tier_read(lmc_tier_t *tier, int32_t dir, const uint64_t *chunk_ids, int64_t n);
int32_t lmc_tier_errno(const lmc_tier_t *tier);
/* files written / bytes written / chunks read back since the tier was opened */
lmc_status_t lmc_tier_get_stats(lmc_tier_t *tier, uint64_t *files_written, uint64_t *bytes_written,
                                uint64_t *chunks_read);

/* LMC_FLAG_EVICT_LRU: the ids evicted since the last call, oldest eviction first, so
 * that a layer above can report them (batched_evict of section 7, Table 3).  Writes at
 * most cap ids to ids_out (HOST) and forgets those; *n_out = how many were written.
 * The log keeps the latest 2^20 evictions. */
lmc_status_t lmc_drain_evicted(lmc_ctx_t *ctx, uint64_t *ids_out, int64_t cap, int64_t *n_out);

lmc_status_t lmc_get_stats(lmc_ctx_t *ctx, lmc_stats_t *out);
lmc_status_t lmc_reset_stats(lmc_ctx_t *ctx);

/* Measurement aids (section 8.6 compares achieved loading bandwidth).
 * lmc_measure_link: best-of-reps hipMemcpyAsync rate between the context's pinned pool
 * and a device buffer, per direction, in GB/s (1e9 bytes/s), for transfers of nbytes
 * (<= pool size).  Blocks.  Pool content is preserved.
 * lmc_copy: a plain device-to-device copy kernel (DEVICE pointers, 16-byte aligned,
 * nbytes a multiple of 16) enqueued on `stream`: the streaming-copy ceiling the
 * gather / scatter kernels are compared with, and the known-size kernel that hardware
 * counters are calibrated on. */
lmc_status_t lmc_measure_link(lmc_ctx_t *ctx, uint64_t nbytes, int32_t reps,
                              double *h2d_gbps_out, double *d2h_gbps_out);
/* The same measurement with the library's link-paced copy kernel (a fixed grid of
 * "link_groups" workgroups reading or writing the pinned pool) in place of the
 * runtime's copy; nbytes a multiple of 16.  The link's peak is the better of the two. */
lmc_status_t lmc_measure_link_kernel(lmc_ctx_t *ctx, uint64_t nbytes, int32_t reps,
                                     double *h2d_gbps_out, double *d2h_gbps_out);
lmc_status_t lmc_copy(lmc_ctx_t *ctx, void *dst_dev, const void *src_dev, uint64_t nbytes,
                      void *stream);
/* The ceiling of an access pattern: a plain copy of 4 KiB tiles in a given order, with no
 * slot mapping and no geometry.  Workgroup w copies tile src_order[w] of src_dev to tile
 * dst_order[w] of dst_dev (tile t = bytes [4096 t, 4096 t + 4096) from the pointer; a NULL
 * order means t = w).  dst_order / src_order: DEVICE uint32[n_tiles]; the caller guarantees
 * that every tile lies inside memory it owns and that no two workgroups write the same tile.
 * Fed with the address stream of a gather or scatter launch it measures what that stream
 * alone costs (section 8.6 compares achieved bandwidths; this is the denominator for the
 * two kernels on a given page placement).  mode 0 copies, 1 only reads, 2 only writes.
 * n_tiles < 2^31.  Enqueued on `stream`. */
lmc_status_t lmc_copy_tiles(lmc_ctx_t *ctx, void *dst_dev, const uint32_t *dst_order,
                            const void *src_dev, const uint32_t *src_order, uint64_t n_tiles,
                            uint32_t mode, void *stream);
/* Both directions at once (section 5.1 "Parallel Store/load Operations": the host link is
 * full duplex): nbytes up and nbytes down at the same time, sum of both directions in
 * GB/s, best of reps.  Needs 2*nbytes of pool; pool content is preserved.  Blocks. */
lmc_status_t lmc_measure_link_duplex(lmc_ctx_t *ctx, uint64_t nbytes, int32_t reps,
                                     double *sum_gbps_out);
/* The same with the library's link-paced copy kernel in place of the runtime's copy for the
 * upload (by_kernel bit 0), the download (bit 1) or both.  Bits 8-15 of by_kernel, if not 0:
 * each direction moves its nbytes as that many consecutive transfers, the way the pipelines
 * issue them group by group.  nbytes a multiple of 16 times the number of pieces.  The
 * two-way peak of the link is the best over the combinations. */
lmc_status_t lmc_measure_link_duplex_kernel(lmc_ctx_t *ctx, uint64_t nbytes, int32_t reps,
                                            uint32_t by_kernel, double *sum_gbps_out);

/* Would work on `stream` (a hipStream_t of the caller, e.g. the stream its model runs on)
 * have to wait behind the library's copies?  HIP maps streams onto a few hardware queues
 * (GPU_MAX_HW_QUEUES, 4 by default) and a queue runs its entries in order, so a stream
 * that shares a queue with one of the library's copy streams stands still while a copy
 * of that stream is under way, whatever the streams' own dependencies say: the overlap
 * of loading with compute (section 5.2) is then lost.  The call enqueues, on each of the
 * library's streams in turn, a copy of up to 64 MiB that only reads the pool, and right
 * behind it an independent small kernel on `stream`; bit i of *mask_out (HOST) is set if
 * that kernel finished only with the copy (bit 0: host-to-device stream, 1: the second
 * one, 2: device-to-host, 3: the second one; bits 4 and 5: the gather and the scatter
 * stream.  Those two count as well: the scatter stream's entries wait for the copies of a
 * retrieve and the gather stream's for those of a store, and under LMC_FLAG_DIRECT the
 * link-paced kernels run there for the length of a transfer.  A stream overlaps with
 * retrieves if bits 0, 1 and 5 are clear, with stores if bits 2, 3 and 4 are).
 * 0 = no sharing: pick such a stream
 * for compute, or raise GPU_MAX_HW_QUEUES so that every stream has a queue of its own.
 * Blocks for some milliseconds; waits for the device first.  LMC_ERR_NOMEM, LMC_ERR_HIP. */
lmc_status_t lmc_probe_stream(lmc_ctx_t *ctx, void *stream, uint32_t *mask_out);

/* Run-time knobs for experiments; the defaults are the measured best.  Keys: "nt_load",
 * "nt_store" (0/1: non-temporal hints on the kernels' streaming accesses), "xcd_run"
 * (consecutive tiles handed to one XCD, 0 = hardware round-robin), "link_groups" (default
 * 64: launches that read or write the pinned pool themselves run as that many workgroups
 * taking tiles in turn, which is what the host link likes; 0 = one tile per workgroup as
 * for launches inside HBM), "copy_kernel" (default 0; bit 0: copies from staging to the
 * pool are made by the library's own link-paced copy kernel instead of hipMemcpyAsync;
 * bit 1: copies from the pool to staging too.  2-3 % slower than the runtime's copies,
 * but independent of which engine the runtime picks and of what else that engine is doing),
 * "d2h_guard" (default 1: the library times the runtime's copies to the host of 32 MiB
 * and more, one per group, and when two of the last four fell below six tenths of the
 * best rate it has seen it makes these copies with its own kernel for 0.25 s, then tries
 * the runtime again, doubling the pause up to 2 s while the runtime stays slow: the
 * runtime's copies to the host lose their rate now and then, for seconds after large
 * allocations and in mixes of stores and retrieves of many requests; 0: never),
 * "edge_chunks" (size
 * of the group at the exposed end of a pipeline, 0 = none), "timing" (0/1: switches
 * LMC_FLAG_TIMING), "trace" (0/1: switches LMC_FLAG_TRACE; 1 also empties the trace and
 * restarts its clock), "direct_store_below" / "direct_retrieve_below" (bytes, default 64 MiB
 * each: an lmc_store with at most that many new bytes, or an lmc_retrieve /
 * lmc_retrieve_batch of at most that many bytes, goes the LMC_FLAG_DIRECT way: one launch
 * instead of kernel, event, copy, event; 0 = never), "scatter_order" (default 0; 1 or 2:
 * scatter launches visit their rows in ascending slot order, built on the device, so that
 * the writes sweep every plane once; 1 = only launches with at least "ordered_min_pages"
 * pages that cover at least one block in "ordered_min_density_inv" of a plane, 2 = every
 * launch; "ordered_group_rows": rows per group, 0 = plane by plane.  Same bytes; on MI355X
 * it measured slower than the plain order at every density, see the benchmark's
 * page_placement figures), "pieces_by_kernel_below" (bytes, default 2 MiB: a group whose
 * chunks lie in several runs of pool slots and whose transfers would average at most that
 * many bytes, i.e. a layer-wise step on a fragmented pool, is copied between staging and
 * pool by one launch of the library's copy kernel instead of one small runtime copy per
 * run; 0 = never), "store_step_streams" (default 2: consecutive lmc_store_layers calls of
 * a ticket put their copies on the two device-to-host copy streams in turn; 1: on one),
 * "caller_waits" (default 1: an lmc_retrieve / lmc_retrieve_batch
 * ends by making the caller's stream wait for it; 0: it does not, and the caller orders its
 * work after the ticket itself with lmc_wait.  A wait that stands at the head of an
 * otherwise idle hardware queue for the length of a large retrieve cost that retrieve
 * 0.5 % on MI355X), "arrange_streams" (1: place the library's streams on hardware queues
 * again, as lmc_create does without LMC_FLAG_KEEP_STREAMS, e.g. after the process has made
 * its own streams; LMC_ERR_BUSY unless every ticket has been waited for),
 * "fail_hip_after" (for tests of the
 * error paths: the n-th HIP call the library checks from now on is not made and counts as
 * failed, once; 0 = off.  Nothing on the device goes wrong).
 * Unknown key or out-of-range value: LMC_ERR_INVAL. */
lmc_status_t lmc_tune(lmc_ctx_t *ctx, const char *key, int64_t value);

/* Component-wise timeline of the pipelines (the paper breaks its delays down by component,
 * sections 8.1 and 8.6; here per step on the device).  Under LMC_FLAG_TRACE every gather
 * launch, every group's device-to-host copies, every group's host-to-device copies and
 * every scatter launch leaves one record when it has completed: kernels with their own
 * begin / end time stamps, copies between two event markers on their copy stream (copies
 * that a fragmented group puts on the second copy stream are inside the same bracket).
 * Times are device time in microseconds since the trace was switched on.  The library keeps
 * the newest 65536 records. */
enum { LMC_STAGE_GATHER = 0, LMC_STAGE_D2H = 1, LMC_STAGE_H2D = 2, LMC_STAGE_SCATTER = 3 };
typedef struct {
    uint64_t ticket;          /* the store / retrieve the step belongs to; 0: lmc_gather / lmc_scatter */
    int32_t stage;            /* LMC_STAGE_* */
    int32_t chunks;           /* chunks of the group */
    uint64_t bytes;           /* payload bytes of the step */
    double begin_us, end_us;
} lmc_trace_rec_t;
/* Takes up to cap finished records out of the trace, oldest first, into out (HOST);
 * *n_out (HOST) receives their number, *dropped_out (HOST, may be NULL) how many records
 * were lost to the limit since the last call.  Steps still running stay for a later call.
 * LMC_ERR_NODEVICE. */
lmc_status_t lmc_trace_read(lmc_ctx_t *ctx, lmc_trace_rec_t *out, int64_t cap, int64_t *n_out,
                            uint64_t *dropped_out);

const char *lmc_strerror(lmc_status_t status);
int32_t lmc_last_hip_error(const lmc_ctx_t *ctx); /* hipError_t of the last LMC_ERR_HIP */

#ifdef __cplusplus
}
#endif
#endif /* LMC_H */
