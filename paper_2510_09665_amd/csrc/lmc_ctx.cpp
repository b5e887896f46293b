// liblmc: the context's life cycle, the chunk index calls, waiting, statistics and tuning
// (see include/lmc.h for the contract; the pipelines are in lmc_pipeline.cpp).
#include "lmc_ctx.hpp"

namespace lmci {

lmc_status_t get_event(lmc_ctx *c, bool timing, hipEvent_t *out) {
    std::vector<hipEvent_t> &pool = timing ? c->free_time_events : c->free_sync_events;
    if (!pool.empty()) {
        *out = pool.back();
        pool.pop_back();
        return LMC_OK;
    }
    hipEvent_t e;
    HIPCHK(c, hipEventCreateWithFlags(&e, timing ? hipEventDefault : hipEventDisableTiming));
    c->all_events.push_back(e);
    *out = e;
    return LMC_OK;
}

static int64_t gcd_pow2(int64_t a, int64_t cap) {
    int64_t v = cap;
    while (v > 1 && (a % v) != 0) v >>= 1;
    return v;
}

// Fill KernelGeom from the public geometry; LMC_ERR_INVAL if it cannot be expressed.
static lmc_status_t derive_geometry(const lmc_kv_geom_t &g, lmc::KernelGeom *k, int64_t *chunk_bytes) {
    if (g.num_layers < 1 || g.num_layers > LMC_MAX_LAYERS || g.num_planes < 1 ||
        g.num_layers * int64_t(g.num_planes) > lmc::kMaxLayerPlanes || g.num_heads < 1 ||
        g.head_dim < 1 || g.elem_bytes < 1 || g.block_size < 1 || g.num_blocks < 1 ||
        g.chunk_tokens < 1)
        return LMC_ERR_INVAL;
    if (g.plane_stride < 0 || g.block_stride < 0 || g.token_stride < 0 || g.head_stride < 0)
        return LMC_ERR_INVAL;
    const int64_t n_slots = int64_t(g.num_blocks) * g.block_size;
    if (n_slots >= (int64_t(1) << 31)) return LMC_ERR_INVAL;
    const int64_t run = int64_t(g.head_dim) * g.elem_bytes;
    const int64_t row = run * g.num_heads;
    if (run >= (int64_t(1) << 31) || row >= (int64_t(1) << 31)) return LMC_ERR_INVAL;
    const bool row_contiguous = (g.num_heads == 1) || (g.head_stride == run);
    int64_t vec = gcd_pow2(run, 16);
    vec = gcd_pow2(g.plane_stride, vec);
    vec = gcd_pow2(g.block_stride, vec);
    vec = gcd_pow2(g.token_stride, vec);
    if (!row_contiguous) vec = gcd_pow2(g.head_stride, vec);
    const int64_t pairs = int64_t(g.chunk_tokens) * (row / vec);
    if (pairs >= (int64_t(1) << 31)) return LMC_ERR_INVAL;

    k->block_stride = g.block_stride;
    k->token_stride = g.token_stride;
    k->run_stride = row_contiguous ? 0 : g.head_stride;
    k->plane_bytes = uint64_t(g.chunk_tokens) * uint64_t(row);
    k->chunk_bytes = k->plane_bytes * uint64_t(g.num_layers) * uint64_t(g.num_planes);
    k->n_slots = uint32_t(n_slots);
    k->chunk_tokens = uint32_t(g.chunk_tokens);
    k->vec_per_plane = uint32_t(pairs);
    k->runs_per_row = row_contiguous ? 1u : uint32_t(g.num_heads);
    k->n_layer_planes = uint32_t(g.num_layers * g.num_planes);
    k->vec = uint32_t(vec);
    k->by_tiles_per_plane = lmc::make_fastdiv(uint32_t((pairs + 255) / 256));
    k->by_vec_per_row = lmc::make_fastdiv(uint32_t(row / vec));
    k->by_vec_per_run = lmc::make_fastdiv(uint32_t((row_contiguous ? row : run) / vec));
    k->by_block_size = lmc::make_fastdiv(uint32_t(g.block_size));
    *chunk_bytes = int64_t(k->chunk_bytes);
    return LMC_OK;
}

lmc_status_t build_layer_ptrs(const lmc_ctx *c, void *const *kv_layers, lmc::LayerPtrs *out) {
    const lmc_kv_geom_t &g = c->cfg.geom;
    for (int l = 0; l < g.num_layers; l++) {
        uint8_t *base = static_cast<uint8_t *>(kv_layers[l]);
        if (base == nullptr || (reinterpret_cast<uintptr_t>(base) % c->kg.vec) != 0)
            return LMC_ERR_INVAL;
        for (int p = 0; p < g.num_planes; p++)
            out->p[l * g.num_planes + p] = base + int64_t(p) * g.plane_stride;
    }
    return LMC_OK;
}

Op *find_op(lmc_ctx *c, uint64_t ticket) {
    for (Op &o : c->ops)
        if (o.ticket == ticket) return &o;
    return nullptr;
}

double seconds_now(const lmc_ctx *c) {
    return std::chrono::duration<double>(std::chrono::steady_clock::now() - c->born).count();
}

// An event without timing that nothing enqueued later will wait on is free again; see
// lmc_ctx::waiters for why it may have to be parked first.
void recycle(lmc_ctx *c, hipEvent_t e) {
    (c->waiters > 0 ? c->held_events : c->free_sync_events).push_back(e);
}

// Finish every operation whose last device step has completed: drop its in-flight
// counts, collect kernel timings, recycle events.
void reap(lmc_ctx *c) {
    for (size_t i = 0; i < c->copy_timings.size();) {
        CopyTiming &t = c->copy_timings[i];
        if (hipEventQuery(t.stop) != hipSuccess) {
            i++;
            continue;
        }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess)
            c->d2h_guard.observe(t.bytes, double(ms) * 1e-3, seconds_now(c));
        c->free_time_events.push_back(t.start);
        c->free_time_events.push_back(t.stop);
        c->copy_timings.erase(c->copy_timings.begin() + long(i));
    }
    c->stats.d2h_guard_switches = c->d2h_guard.switches();
    c->stats.d2h_guard_active = (c->d2h_guard_on && c->d2h_guard.use_kernel(seconds_now(c))) ? 1 : 0;
    c->stats.d2h_copy_best_gbps = c->d2h_guard.best_rate() * 1e-9;
    c->stats.d2h_copy_last_gbps = c->d2h_guard.last_rate() * 1e-9;
    for (size_t i = 0; i < c->ops.size();) {
        Op &op = c->ops[i];
        const bool finished = op.done != nullptr ? hipEventQuery(op.done) == hipSuccess : !op.pending;
        if (!finished) {
            i++;
            continue;
        }
        if (op.done != nullptr) recycle(c, op.done);
        for (hipEvent_t e : op.owned_events) recycle(c, e);
        for (int64_t s : op.slots) {
            lmc::SlotMeta &m = c->index.meta(s);
            m.inflight--;
            if (m.ready_ticket == op.ticket) {
                m.ready_ticket = 0;
                m.ready_event = nullptr;
            }
        }
        c->ops.erase(c->ops.begin() + long(i));
    }
    for (size_t i = 0; i < c->timings.size();) {
        Timing &t = c->timings[i];
        if (hipEventQuery(t.stop) == hipSuccess) {
            float ms = 0.f;
            const bool kernel = t.stage == LMC_STAGE_GATHER || t.stage == LMC_STAGE_SCATTER;
            if (kernel && hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
                if (t.stage == LMC_STAGE_GATHER) {
                    c->stats.gather_ms += ms;
                    c->stats.timed_gather_launches++;
                } else {
                    c->stats.scatter_ms += ms;
                    c->stats.timed_scatter_launches++;
                }
            }
            float b = 0.f, e = 0.f;
            if ((c->cfg.flags & LMC_FLAG_TRACE) && c->trace_epoch != nullptr &&
                hipEventElapsedTime(&b, c->trace_epoch, t.start) == hipSuccess &&
                hipEventElapsedTime(&e, c->trace_epoch, t.stop) == hipSuccess) {
                if (c->trace.size() >= kTraceCap) {
                    c->trace.pop_front();
                    c->trace_dropped++;
                }
                c->trace.push_back(lmc_trace_rec_t{t.ticket, t.stage, t.chunks, t.bytes, double(b) * 1e3, double(e) * 1e3});
            }
            c->free_time_events.push_back(t.start);
            c->free_time_events.push_back(t.stop);
            c->timings.erase(c->timings.begin() + long(i));
        } else {
            i++;
        }
    }
    (void)hipGetLastError();
}

// LMC_FLAG_TRACE: a timing event in front of the copies of a group ...
lmc_status_t trace_begin(lmc_ctx *c, hipStream_t stream, hipEvent_t *start) {
    *start = nullptr;
    if (!(c->cfg.flags & LMC_FLAG_TRACE)) return LMC_OK;
    lmc_status_t rc = get_event(c, true, start);
    if (rc != LMC_OK) return rc;
    const hipError_t e = injected_failure(c) ? hipErrorUnknown : hipEventRecord(*start, stream);
    if (e != hipSuccess) {
        c->free_time_events.push_back(*start);
        *start = nullptr;
        HIPCHK(c, e);
    }
    return LMC_OK;
}

// ... and one behind them; the pair is read when both have completed (reap).
lmc_status_t trace_end(lmc_ctx *c, hipStream_t stream, hipEvent_t start, int32_t stage, int64_t chunks, uint64_t bytes) {
    if (start == nullptr) return LMC_OK;
    hipEvent_t stop = nullptr;
    lmc_status_t rc = get_event(c, true, &stop);
    hipError_t e = hipSuccess;
    if (rc == LMC_OK) e = injected_failure(c) ? hipErrorUnknown : hipEventRecord(stop, stream);
    if (rc != LMC_OK || e != hipSuccess) {
        c->free_time_events.push_back(start);
        if (stop) c->free_time_events.push_back(stop);
        if (rc != LMC_OK) return rc;
        HIPCHK(c, e);
    }
    c->timings.push_back(Timing{start, stop, stage, c->cur_ticket, int32_t(chunks), bytes});
    return LMC_OK;
}

// Orders `waiter` after everything enqueued so far on `stream`.
lmc_status_t order_after(lmc_ctx *c, hipStream_t waiter, hipStream_t stream) {
    hipEvent_t e;
    lmc_status_t rc = get_event(c, false, &e);
    if (rc != LMC_OK) return rc;
    HIPCHK(c, hipEventRecord(e, stream));
    HIPCHK(c, hipStreamWaitEvent(waiter, e, 0));
    // the event can be reused once recorded again: waits already enqueued keep the
    // record they saw
    c->free_sync_events.push_back(e);
    return LMC_OK;
}

// Orders `waiter` after the work the caller has put on its own stream so far.  A stream
// with nothing pending needs no event, and is better off without one: an event recorded on
// the caller's stream takes its place in that stream's hardware queue, behind whatever a
// library stream that shares the queue still has to run (with a store under way and the
// caller's stream in the gather stream's queue, a retrieve issued next would start only
// when the store's last gather has run).  This holds for the null stream too: work recorded
// there also waits for what the process's other blocking streams hold, and the runtime's
// query of the null stream answers "not ready" while any of them is busy (checked by
// tests/test_gpu_streams.py, with the producer of the KV on a blocking stream).
lmc_status_t order_after_caller(lmc_ctx *c, hipStream_t waiter, hipStream_t user) {
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(user, &capturing) == hipSuccess && capturing == hipStreamCaptureStatusNone) {
        if (hipStreamQuery(user) == hipSuccess) return LMC_OK;
    }
    (void)hipGetLastError();   // "not ready" is an answer, not a failure
    return order_after(c, waiter, user);
}

// Is an operation of the other direction still under way?  The second copy stream of a
// direction sits in the hardware queue of the other direction's kernel stream (see
// arrange_streams), and as created any two streams may share one: next to a transfer the
// other way a second copy stream would not add a copy in flight but hold that transfer's
// kernels or copies up, so it is left out then.
bool other_direction_busy(lmc_ctx *c, bool for_store) {
    for (const Op &o : c->ops) {
        const bool is_store = o.pending || o.final_stream == c->s_d2h || o.final_stream == c->s_d2h2 || o.final_stream == c->s_gather;
        if (is_store == for_store) continue;
        if (o.pending) return true;
        if (o.done != nullptr && hipEventQuery(o.done) != hipSuccess) {
            (void)hipGetLastError();
            return true;
        }
    }
    return false;
}

// LMC_FLAG_VALIDATE_SLOTS: device-side range check with a host wait.
lmc_status_t validate_slots(lmc_ctx *c, const int64_t *slot_mapping, int64_t n_tokens,
                            hipStream_t stream) {
    if (!(c->cfg.flags & LMC_FLAG_VALIDATE_SLOTS) || n_tokens == 0) return LMC_OK;
    // the check has a flag word of its own (kCheckWord): the shared one may be set at any
    // moment by a kernel of an earlier call that is still running, and that report
    // belongs to the next lmc_wait, not to this call
    HIPCHK(c, hipStreamSynchronize(stream));
    c->bad_flag_host[kCheckWord] = 0;
    HIPCHK(c, lmc::launch_check_slots(slot_mapping, uint64_t(n_tokens), c->kg.n_slots,
                                      c->bad_flag_dev + kCheckWord, stream));
    HIPCHK(c, hipStreamSynchronize(stream));
    return c->bad_flag_host[kCheckWord] != 0 ? LMC_ERR_BADSLOT : LMC_OK;
}

lmc_status_t force_sync(lmc_ctx *c, hipStream_t s) {
    if (c->cfg.flags & LMC_FLAG_FORCE_SYNC) HIPCHK(c, hipStreamSynchronize(s));
    return LMC_OK;
}

lmc_status_t free_ring(Ring &r) {
    for (uint8_t *p : r.buf)
        if (p) (void)hipFree(p);
    r.buf.clear();
    return LMC_OK;
}

lmc_status_t make_ring(lmc_ctx *c, Ring &r) {
    const size_t n = size_t(c->cfg.num_staging);
    r.buf_bytes = uint64_t(c->cfg.staging_chunks) * uint64_t(c->chunk_bytes);
    r.buf.assign(n, nullptr);
    for (size_t i = 0; i < n; i++) {
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&r.buf[i]), r.buf_bytes);
        if (e != hipSuccess) {
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
            return e == hipErrorOutOfMemory ? LMC_ERR_NOMEM : LMC_ERR_HIP;
        }
    }
    return LMC_OK;
}

// Recency of use.  A call that uses chunks takes the next call number and stamps the
// chunks it finds present (they are then safe from the call's own evictions) ...
void begin_use(lmc_ctx *c, const uint64_t *ids, int64_t n) {
    c->use_calls++;
    for (int64_t i = 0; i < n; i++) {
        const int64_t s = c->index.find(ids[i]);
        if (s >= 0) c->index.meta(s).use_call = c->use_calls;
    }
}

// ... and when it ends its chunks become the newest, the first of the call the newest of
// all: within a call the later position is the older one, so a request loses its tail
// before its head and what is left still hits as a prefix.
void end_use(lmc_ctx *c, const uint64_t *ids, int64_t n) {
    for (int64_t i = n - 1; i >= 0; i--) {
        const int64_t s = c->index.find(ids[i]);
        if (s >= 0) c->index.touch(s);
    }
}

// Sleeps until every event of `evs` has completed, with the context's mutex released so
// that other threads go on storing, loading and looking up meanwhile.  The events stay
// valid: whatever reap() frees while somebody sleeps is parked (lmc_ctx::waiters).
static lmc_status_t sync_unlocked(lmc_ctx *c, std::unique_lock<std::mutex> &lock,
                           const std::vector<hipEvent_t> &evs) {
    if (evs.empty()) return LMC_OK;
    c->waiters++;
    lock.unlock();
    hipError_t err = hipSuccess;
    for (hipEvent_t e : evs) {
        const hipError_t x = hipEventSynchronize(e);
        if (x != hipSuccess && err == hipSuccess) err = x;
    }
    lock.lock();
    if (--c->waiters == 0) {
        c->free_sync_events.insert(c->free_sync_events.end(), c->held_events.begin(), c->held_events.end());
        c->held_events.clear();
    }
    if (err != hipSuccess) {
        c->last_hip_error = int32_t(err);
        (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
        return LMC_ERR_HIP;
    }
    return LMC_OK;
}

// The store that fills the slot of chunk `id`, if it is still under way: the event behind
// the copies of the chunk's group, or else the store's last event, goes to *ev (null =
// nothing to wait for).  LMC_ERR_MISS / LMC_ERR_BUSY as lmc_get_host.
static lmc_status_t pending_fill(lmc_ctx *c, uint64_t id, int64_t *slot_out, hipEvent_t *ev) {
    *ev = nullptr;
    const int64_t s = c->index.find(id);
    if (s < 0) return LMC_ERR_MISS;
    *slot_out = s;
    const lmc::SlotMeta &m = c->index.meta(s);
    if (m.ready_ticket != 0) {
        const Op *o = find_op(c, m.ready_ticket);
        if (o != nullptr && o->pending) return LMC_ERR_BUSY;
        if (o != nullptr) *ev = m.ready_event != nullptr ? static_cast<hipEvent_t>(m.ready_event) : o->done;
    }
    return LMC_OK;
}

// Switches the trace on: device time counts from here.
static lmc_status_t start_trace(lmc_ctx *c) {
    if (c->trace_epoch == nullptr) {
        lmc_status_t rc = get_event(c, true, &c->trace_epoch);
        if (rc != LMC_OK) return rc;
    }
    HIPCHK(c, hipEventRecord(c->trace_epoch, c->s_gather));
    HIPCHK(c, hipEventSynchronize(c->trace_epoch));
    c->trace.clear();
    c->trace_dropped = 0;
    c->cfg.flags |= LMC_FLAG_TRACE;
    return LMC_OK;
}

static void destroy_ctx(lmc_ctx *c) {
    if (c->has_device) {
        DeviceScope dev(c);
        (void)hipDeviceSynchronize();
        free_ring(c->store_ring);
        free_ring(c->load_ring);
        for (void *p : {static_cast<void *>(c->order.token_at), static_cast<void *>(c->order.counts),
                        static_cast<void *>(c->order.n_rows), static_cast<void *>(c->order.pairs)})
            if (p) (void)hipFree(p);
        for (void *p : c->order_retired) (void)hipFree(p);
        for (hipEvent_t e : c->all_events) (void)hipEventDestroy(e);
        for (hipStream_t s : {c->s_gather, c->s_d2h, c->s_h2d, c->s_scatter, c->s_h2d2, c->s_d2h2})
            if (s) (void)hipStreamDestroy(s);
        if (c->bad_flag_host) (void)hipHostFree(c->bad_flag_host);
        if (c->pool) (void)hipHostFree(c->pool);
    } else {
        std::free(c->pool);
    }
    delete c;
}

// A slot for a new chunk: the lowest free one; with LMC_FLAG_EVICT_LRU and a full pool
// the least recently used chunk that may go gives up its slot.  -1: no room.
int64_t take_slot(lmc_ctx *c, uint64_t id) {
    int64_t s = c->index.insert(id);
    if (s < 0 && (c->cfg.flags & LMC_FLAG_EVICT_LRU)) {
        const int64_t v = c->index.victim(c->use_calls);
        if (v >= 0) {
            const uint64_t gone = c->index.meta(v).id;
            c->index.erase(gone);
            c->stats.chunks_evicted++;
            if (c->evicted.size() >= (size_t(1) << 20))
                c->evicted.erase(c->evicted.begin(), c->evicted.begin() + (size_t(1) << 19));
            c->evicted.push_back(gone);
            s = c->index.insert(id);
        }
    }
    if (s < 0) c->stats.alloc_failures++;
    else c->index.meta(s).use_call = c->use_calls;
    return s;
}

}  // namespace lmci

using namespace lmci;

extern "C" {

lmc_status_t lmc_create(const lmc_config_t *cfg, lmc_ctx_t **ctx_out) {
    if (!cfg || !ctx_out) return LMC_ERR_INVAL;
    *ctx_out = nullptr;
    lmc_ctx *c = new (std::nothrow) lmc_ctx();
    if (!c) return LMC_ERR_NOMEM;
    c->cfg = *cfg;
    lmc_status_t rc = derive_geometry(cfg->geom, &c->kg, &c->chunk_bytes);
    if (rc == LMC_OK && (cfg->num_staging < 2 || cfg->staging_chunks < 1 ||
                         (cfg->device < 0 && cfg->device != LMC_DEVICE_NONE)))
        rc = LMC_ERR_INVAL;
    if (rc == LMC_OK) {
        c->n_pool_slots = int64_t(cfg->host_pool_bytes / uint64_t(c->chunk_bytes));
        if (c->n_pool_slots < 1) rc = LMC_ERR_INVAL;
        // one launch must be able to cover a whole staging buffer
        if (int64_t(cfg->staging_chunks) > int64_t(lmc::max_chunks_per_launch(c->kg, lmc::bulk_view(c->kg))))
            rc = LMC_ERR_INVAL;
    }
    if (rc != LMC_OK) {
        delete c;
        return rc;
    }
    c->shape.nt_load = true;
    c->shape.nt_store = true;
    c->shape.xcd_run = 32;
    c->shape.paced_groups = 0;
    c->shape.ordered_group_rows = 256;
    c->has_device = cfg->device != LMC_DEVICE_NONE;
    const size_t pool_bytes = size_t(c->n_pool_slots) * size_t(c->chunk_bytes);
    if (!c->has_device) {
        c->pool = static_cast<uint8_t *>(std::aligned_alloc(4096, (pool_bytes + 4095) / 4096 * 4096));
        if (!c->pool) {
            delete c;
            return LMC_ERR_NOMEM;
        }
    } else {
        int n_dev = 0;
        hipError_t e = hipGetDeviceCount(&n_dev);
        if (e != hipSuccess || cfg->device >= n_dev) {
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
            delete c;
            return e != hipSuccess ? LMC_ERR_HIP : LMC_ERR_INVAL;
        }
        DeviceScope dev(c);
        auto fail = [&](lmc_status_t st) {
            destroy_ctx(c);
            return st;
        };
        e = hipHostMalloc(reinterpret_cast<void **>(&c->pool), pool_bytes, hipHostMallocDefault);
        if (e != hipSuccess) {
            c->pool = nullptr;
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
            return fail(LMC_ERR_NOMEM);
        }
        if (hipHostGetDevicePointer(reinterpret_cast<void **>(&c->pool_dev), c->pool, 0) != hipSuccess)
            return fail(LMC_ERR_HIP);
        e = hipHostMalloc(reinterpret_cast<void **>(&c->bad_flag_host), 64, hipHostMallocMapped);
        if (e != hipSuccess) {
            c->bad_flag_host = nullptr;
            return fail(LMC_ERR_HIP);
        }
        std::memset(c->bad_flag_host, 0, 64);
        if (hipHostGetDevicePointer(reinterpret_cast<void **>(&c->bad_flag_dev), c->bad_flag_host, 0) != hipSuccess)
            return fail(LMC_ERR_HIP);
        for (hipStream_t *s : {&c->s_gather, &c->s_d2h, &c->s_h2d, &c->s_scatter, &c->s_h2d2, &c->s_d2h2})
            if (hipStreamCreateWithFlags(s, hipStreamNonBlocking) != hipSuccess) return fail(LMC_ERR_HIP);
        if ((e = resolve_static_scratch(cfg->device)) != hipSuccess) {
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();
            return fail(LMC_ERR_HIP);
        }
        if ((rc = make_ring(c, c->store_ring)) != LMC_OK) return fail(rc);
        if ((rc = make_ring(c, c->load_ring)) != LMC_OK) return fail(rc);
        if (!(cfg->flags & LMC_FLAG_KEEP_STREAMS)) arrange_streams(c);
        if ((cfg->flags & LMC_FLAG_TRACE) && (rc = start_trace(c)) != LMC_OK) return fail(rc);
    }
    c->index.reset(c->n_pool_slots);
    c->stats.pool_slots_total = uint64_t(c->n_pool_slots);
    *ctx_out = c;
    return LMC_OK;
}

lmc_status_t lmc_destroy(lmc_ctx_t *c) {
    if (!c) return LMC_ERR_INVAL;
    destroy_ctx(c);
    return LMC_OK;
}

int64_t lmc_chunk_bytes(const lmc_ctx_t *c) { return c ? c->chunk_bytes : 0; }

int32_t lmc_chunk_tokens(const lmc_ctx_t *c) { return c ? c->cfg.geom.chunk_tokens : 0; }

int32_t lmc_block_size(const lmc_ctx_t *c) { return c ? c->cfg.geom.block_size : 0; }

int64_t lmc_pool_slots(const lmc_ctx_t *c) { return c ? c->n_pool_slots : 0; }

lmc_status_t lmc_hash_chunks_from(const lmc_ctx_t *c, uint64_t prev_id, const int32_t *tokens,
                                  int64_t n_tokens, uint64_t *ids_out, int64_t *n_chunks_out) {
    if (!c || n_tokens < 0 || (n_tokens > 0 && !tokens) || !n_chunks_out) return LMC_ERR_INVAL;
    const int32_t CT = c->cfg.geom.chunk_tokens;
    const int64_t n = n_tokens / CT;
    if (n > 0 && !ids_out) return LMC_ERR_INVAL;
    uint64_t prev = prev_id;
    for (int64_t i = 0; i < n; i++) {
        prev = lmc::chunk_id(prev, tokens + i * CT, CT);
        ids_out[i] = prev;
    }
    *n_chunks_out = n;
    return LMC_OK;
}

lmc_status_t lmc_hash_chunks(const lmc_ctx_t *c, const int32_t *tokens, int64_t n_tokens,
                             uint64_t *ids_out, int64_t *n_chunks_out) {
    if (!c) return LMC_ERR_INVAL;
    return lmc_hash_chunks_from(c, c->cfg.hash_seed, tokens, n_tokens, ids_out, n_chunks_out);
}

lmc_status_t lmc_lookup(lmc_ctx_t *c, const uint64_t *ids, int64_t n, int64_t *n_hit_out) {
    if (!c || n < 0 || (n > 0 && !ids) || !n_hit_out) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    int64_t k = 0;
    while (k < n && c->index.find(ids[k]) >= 0) k++;
    *n_hit_out = k;
    return LMC_OK;
}

lmc_status_t lmc_wait(lmc_ctx_t *c, uint64_t ticket) {
    if (!c) return LMC_ERR_INVAL;
    std::unique_lock<std::mutex> lock(c->mu);
    const bool everything = ticket == 0;
    if (everything) ticket = c->next_ticket - 1;
    if (ticket >= c->next_ticket) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_OK;
    DeviceScope dev(c);
    // Operations end on different streams that are not ordered among each other (a staged
    // store on the D2H stream, a store without staging on the gather stream, every
    // retrieve on the scatter stream), so the newest operation alone says nothing about
    // the older ones: the newest event of every such stream is waited for.
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> last;
    for (const Op &o : c->ops) {
        if (o.ticket > ticket) continue;
        if (o.pending) {
            // a layer-wise store still short of layers cannot be waited for; when it is
            // merely older than the ticket asked for, it is left out
            if (everything || o.ticket == ticket) return LMC_ERR_BUSY;
            continue;
        }
        if (o.done == nullptr) continue;
        const size_t i = size_t(std::find(streams.begin(), streams.end(), o.final_stream) - streams.begin());
        if (i == streams.size()) {
            streams.push_back(o.final_stream);
            last.push_back(o.done);
        } else {
            last[i] = o.done;   // c->ops is in ticket order, and a stream finishes in order
        }
    }
    const lmc_status_t rc = sync_unlocked(c, lock, last);
    if (rc != LMC_OK) return rc;
    reap(c);
    if (*c->bad_flag_host != 0) {
        *c->bad_flag_host = 0;
        return LMC_ERR_BADSLOT;
    }
    return LMC_OK;
}

lmc_status_t lmc_test(lmc_ctx_t *c, uint64_t ticket) {
    if (!c || ticket == 0) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    if (ticket >= c->next_ticket) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_OK;
    DeviceScope dev(c);
    reap(c);
    return find_op(c, ticket) == nullptr ? LMC_OK : LMC_ERR_BUSY;
}

lmc_status_t lmc_put_host(lmc_ctx_t *c, const uint64_t *ids, int64_t n, const void *host_src) {
    if (!c || n < 0 || (n > 0 && (!ids || !host_src))) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    const uint8_t *src = static_cast<const uint8_t *>(host_src);
    lmc_status_t rc = LMC_OK;
    begin_use(c, ids, n);
    for (int64_t i = 0; i < n; i++) {
        if (c->index.find(ids[i]) >= 0) {
            c->stats.chunks_skipped_dup++;
            continue;
        }
        const int64_t s = take_slot(c, ids[i]);
        if (s < 0) {
            rc = LMC_ERR_NOMEM;
            break;
        }
        std::memcpy(c->pool + s * c->chunk_bytes, src + i * c->chunk_bytes, size_t(c->chunk_bytes));
        c->stats.chunks_stored++;
    }
    end_use(c, ids, n);
    return rc;
}

lmc_status_t lmc_drain_evicted(lmc_ctx_t *c, uint64_t *ids_out, int64_t cap, int64_t *n_out) {
    if (!c || cap < 0 || !n_out || (cap > 0 && !ids_out)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    const size_t n = std::min(c->evicted.size(), size_t(cap));
    std::copy(c->evicted.begin(), c->evicted.begin() + long(n), ids_out);
    c->evicted.erase(c->evicted.begin(), c->evicted.begin() + long(n));
    *n_out = int64_t(n);
    return LMC_OK;
}

lmc_status_t lmc_get_host(lmc_ctx_t *c, uint64_t id, void *host_dst) {
    if (!c || !host_dst) return LMC_ERR_INVAL;
    std::unique_lock<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    // the bytes must have arrived: wait, without holding up other threads, for the store
    // that fills the slot; the chunk may be gone when this thread is back
    for (;;) {
        int64_t s = -1;
        hipEvent_t ev = nullptr;
        lmc_status_t rc = pending_fill(c, id, &s, &ev);
        if (rc != LMC_OK) return rc;
        if (ev == nullptr || hipEventQuery(ev) == hipSuccess) {
            std::memcpy(host_dst, c->pool + s * c->chunk_bytes, size_t(c->chunk_bytes));
            return LMC_OK;
        }
        if ((rc = sync_unlocked(c, lock, {ev})) != LMC_OK) return rc;
        reap(c);
    }
}

lmc_status_t lmc_chunk_acquire(lmc_ctx_t *c, uint64_t id, const void **host_ptr_out) {
    if (!c || !host_ptr_out) return LMC_ERR_INVAL;
    std::unique_lock<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    for (;;) {
        int64_t s = -1;
        hipEvent_t ev = nullptr;
        lmc_status_t rc = pending_fill(c, id, &s, &ev);
        if (rc != LMC_OK) return rc;
        if (ev == nullptr || hipEventQuery(ev) == hipSuccess) {
            c->index.meta(s).refs++;
            *host_ptr_out = c->pool + s * c->chunk_bytes;
            return LMC_OK;
        }
        if ((rc = sync_unlocked(c, lock, {ev})) != LMC_OK) return rc;
        reap(c);
    }
}

lmc_status_t lmc_chunk_release(lmc_ctx_t *c, uint64_t id) {
    if (!c) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    const int64_t s = c->index.find(id);
    if (s < 0) return LMC_ERR_MISS;
    if (c->index.meta(s).refs == 0) return LMC_ERR_INVAL;
    c->index.meta(s).refs--;
    return LMC_OK;
}

lmc_status_t lmc_find_slot(lmc_ctx_t *c, uint64_t id, int64_t *slot_out) {
    if (!c || !slot_out) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    const int64_t s = c->index.find(id);
    if (s < 0) return LMC_ERR_MISS;
    *slot_out = s;
    return LMC_OK;
}

lmc_status_t lmc_pin(lmc_ctx_t *c, const uint64_t *ids, int64_t n) {
    if (!c || n < 0 || (n > 0 && !ids)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    for (int64_t i = 0; i < n; i++)
        if (c->index.find(ids[i]) < 0) return LMC_ERR_MISS;
    for (int64_t i = 0; i < n; i++) c->index.meta(c->index.find(ids[i])).pins++;
    return LMC_OK;
}

lmc_status_t lmc_unpin(lmc_ctx_t *c, const uint64_t *ids, int64_t n) {
    if (!c || n < 0 || (n > 0 && !ids)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    for (int64_t i = 0; i < n; i++)
        if (c->index.find(ids[i]) < 0) return LMC_ERR_MISS;
    // take the pins one by one; if one is missing, give back what was taken
    for (int64_t i = 0; i < n; i++) {
        lmc::SlotMeta &m = c->index.meta(c->index.find(ids[i]));
        if (m.pins == 0) {
            for (int64_t j = 0; j < i; j++) c->index.meta(c->index.find(ids[j])).pins++;
            return LMC_ERR_INVAL;
        }
        m.pins--;
    }
    return LMC_OK;
}

lmc_status_t lmc_clear(lmc_ctx_t *c, const uint64_t *ids, int64_t n) {
    if (!c || n < 0 || (n > 0 && !ids)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    for (int64_t i = 0; i < n; i++) {
        const int64_t s = c->index.find(ids[i]);
        if (s < 0) continue;
        const lmc::SlotMeta &m = c->index.meta(s);
        if (m.pins > 0 || m.inflight > 0 || m.refs > 0) return LMC_ERR_BUSY;
    }
    for (int64_t i = 0; i < n; i++) c->index.erase(ids[i]);
    return LMC_OK;
}

lmc_status_t lmc_get_stats(lmc_ctx_t *c, lmc_stats_t *out) {
    if (!c || !out) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    c->stats.pool_slots_used = uint64_t(c->index.used());
    *out = c->stats;
    return LMC_OK;
}

lmc_status_t lmc_reset_stats(lmc_ctx_t *c) {
    if (!c) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->has_device) reap(c);
    const uint64_t total = c->stats.pool_slots_total;
    c->stats = lmc_stats_t{};
    c->stats.pool_slots_total = total;
    return LMC_OK;
}

lmc_status_t lmc_trace_read(lmc_ctx_t *c, lmc_trace_rec_t *out, int64_t cap, int64_t *n_out, uint64_t *dropped_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !out)) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    reap(c);
    int64_t n = 0;
    while (n < cap && !c->trace.empty()) {
        out[n++] = c->trace.front();
        c->trace.pop_front();
    }
    *n_out = n;
    if (dropped_out) {
        *dropped_out = c->trace_dropped;
        c->trace_dropped = 0;
    }
    return LMC_OK;
}

lmc_status_t lmc_tune(lmc_ctx_t *c, const char *key, int64_t value) {
    if (!c || !key || value < 0) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    const std::string k(key);
    if (k == "timing" && value <= 1) {
        c->cfg.flags = value ? (c->cfg.flags | LMC_FLAG_TIMING) : (c->cfg.flags & ~LMC_FLAG_TIMING);
    } else if (k == "trace" && value <= 1) {
        if (!c->has_device) return LMC_ERR_NODEVICE;
        if (value == 0) {
            c->cfg.flags &= ~LMC_FLAG_TRACE;
        } else {
            DeviceScope dev(c);
            lmc_status_t rc = start_trace(c);
            if (rc != LMC_OK) return rc;
        }
    } else if (k == "edge_chunks") {
        c->edge_chunks = value;
    } else if (k == "direct_store_below") {
        c->direct_store_below = value;
    } else if (k == "direct_retrieve_below") {
        c->direct_retrieve_below = value;
    } else if (k == "xcd_run") {
        if (value > (1 << 20)) return LMC_ERR_INVAL;
        c->shape.xcd_run = uint32_t(value);
    } else if (k == "d2h_guard" && value <= 1) {
        c->d2h_guard_on = value != 0;
    } else if (k == "store_step_streams" && value >= 1 && value <= 2) {
        c->store_step_streams = int32_t(value);
    } else if (k == "pieces_by_kernel_below") {
        c->pieces_by_kernel_below = uint64_t(value);
    } else if (k == "caller_waits" && value <= 1) {
        c->caller_waits = value != 0;
    } else if (k == "copy_kernel" && value <= 3) {
        c->copy_kernel = uint32_t(value);
    } else if (k == "link_groups") {
        if (value > 65536) return LMC_ERR_INVAL;
        c->link_groups = uint32_t(value);
    } else if (k == "scatter_order" && value <= 2) {
        c->scatter_order = int32_t(value);
    } else if (k == "ordered_group_rows" && value < (int64_t(1) << 31)) {
        c->shape.ordered_group_rows = uint32_t(value);
    } else if (k == "ordered_min_pages") {
        c->ordered_min_pages = value;
    } else if (k == "ordered_min_density_inv" && value >= 1) {
        c->ordered_min_density_inv = value;
    } else if (k == "arrange_streams" && value == 1) {
        if (!c->has_device) return LMC_ERR_NODEVICE;
        if (!c->ops.empty() || !c->held_events.empty()) return LMC_ERR_BUSY;
        DeviceScope dev(c);
        arrange_streams(c);
    } else if (k == "fail_hip_after") {
        if (value > 0xFFFFFFFFll) return LMC_ERR_INVAL;
        c->fail_hip_after = uint32_t(value);
    } else if (k == "nt_load" && value <= 1) {
        c->shape.nt_load = value != 0;
    } else if (k == "nt_store" && value <= 1) {
        c->shape.nt_store = value != 0;
    } else {
        return LMC_ERR_INVAL;
    }
    return LMC_OK;
}

const char *lmc_strerror(lmc_status_t s) {
    switch (s) {
        case LMC_OK: return "ok";
        case LMC_ERR_INVAL: return "invalid argument";
        case LMC_ERR_NOMEM: return "out of memory / pool full";
        case LMC_ERR_MISS: return "chunk not present";
        case LMC_ERR_BADSLOT: return "slot outside the paged KV memory";
        case LMC_ERR_HIP: return "HIP call failed";
        case LMC_ERR_BUSY: return "chunk pinned or in flight";
        case LMC_ERR_IO: return "file input / output failed";
        case LMC_ERR_NODEVICE: return "context has no device";
    }
    return "unknown status";
}

int32_t lmc_last_hip_error(const lmc_ctx_t *c) { return c ? c->last_hip_error : 0; }

}  // extern "C"
