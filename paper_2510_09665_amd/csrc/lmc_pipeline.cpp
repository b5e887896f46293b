// liblmc: the store and retrieve pipelines (see include/lmc.h for the contract).
//
// Store  (paper sections 4 and 5.1): index probe -> per group of new chunks
//        gather kernel (stream G) -> event -> hipMemcpyAsync D2H into pool slots
//        (stream D) -> event that releases the staging buffer.
// Retrieve: hipMemcpyAsync H2D of the hit chunks (stream H) -> event -> scatter kernel
//        (stream S) -> event that releases the staging buffer.
// Each direction owns a ring of num_staging buffers, so the kernel of group k+1 runs
// while the copy of group k is on the link (section 1 (#1): storing and loading are
// batched and pipelined).  The host never waits inside store / retrieve; control
// crosses to the device once per group and direction, not once per page, which is
// the paper's argument for chunk-granular transfers (section 8.6, Table 5).
#include "lmc_ctx.hpp"

namespace lmci {

// Does this scatter launch go in the order of the destination?  It pays when the launch
// finds neighbours among its pages: many pages per plane, and a fair share of the plane.
static bool use_ordered_scatter(const lmc_ctx *c, const lmc::LaunchView &view, uint64_t n_tokens) {
    if (c->scatter_order == 0 || !lmc::ordered_scatter_fits(c->kg, view, c->shape, n_tokens)) return false;
    if (c->scatter_order >= 2) return true;
    const int64_t pages = int64_t(n_tokens) / c->cfg.geom.block_size;
    return pages >= c->ordered_min_pages && pages * c->ordered_min_density_inv >= int64_t(c->cfg.geom.num_blocks);
}

// The scratch of an ordered launch: allocated when first needed, grown when a launch has
// more tokens than any before (the outgrown arrays may still be in use by a launch under
// way and are kept until the context goes).  `stream` is made to wait for the previous
// ordered launch, which may have run on another stream: one set serves one launch at a time.
static lmc_status_t prepare_order_scratch(lmc_ctx *c, uint64_t n_tokens, hipStream_t stream) {
    auto alloc = [&](void **p, uint64_t bytes) -> lmc_status_t {
        const hipError_t e = injected_failure(c) ? hipErrorOutOfMemory : hipMalloc(p, bytes);
        if (e != hipSuccess) {
            *p = nullptr;
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();
            return e == hipErrorOutOfMemory ? LMC_ERR_NOMEM : LMC_ERR_HIP;
        }
        return LMC_OK;
    };
    lmc_status_t rc = LMC_OK;
    if (c->order.token_at == nullptr) {
        void *a = nullptr, *b = nullptr, *n = nullptr;
        rc = alloc(&a, lmc::order_table_words(c->kg) * 4);
        if (rc == LMC_OK) rc = alloc(&b, lmc::order_count_words(c->kg) * 4);
        if (rc == LMC_OK) rc = alloc(&n, 256);
        if (rc == LMC_OK) rc = get_event(c, false, &c->order_free);
        if (rc != LMC_OK) {
            for (void *p : {a, b, n})
                if (p) (void)hipFree(p);
            return rc;
        }
        c->order.token_at = static_cast<uint32_t *>(a);
        c->order.counts = static_cast<uint32_t *>(b);
        c->order.n_rows = static_cast<uint32_t *>(n);
    } else if (c->order_cap_tokens > 0) {
        HIPCHK(c, hipStreamWaitEvent(stream, c->order_free, 0));
    }
    if (n_tokens > c->order_cap_tokens) {
        void *p = nullptr;
        const uint64_t cap = std::max<uint64_t>(n_tokens, 2 * c->order_cap_tokens);
        if ((rc = alloc(&p, cap * 8)) != LMC_OK) return rc;
        if (c->order.pairs != nullptr) c->order_retired.push_back(c->order.pairs);
        c->order.pairs = static_cast<uint2 *>(p);
        c->order_cap_tokens = cap;
    }
    return LMC_OK;
}

lmc_status_t timed_launch(lmc_ctx *c, bool gather, const lmc::LaunchView &view,
                          const lmc::LayerPtrs &ptrs, const int64_t *slots, uint32_t n_chunks,
                          uint8_t *staging, hipStream_t stream) {
    // LMC_FLAG_TIMING: the launch itself carries a start and a stop event, which receive
    // the kernel's own begin / end time stamps; the stream gets no extra marker.
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->cfg.flags & (LMC_FLAG_TIMING | LMC_FLAG_TRACE)) {
        lmc_status_t rc = get_event(c, true, &e0);
        if (rc == LMC_OK) rc = get_event(c, true, &e1);
        if (rc != LMC_OK) return rc;
    }
    lmc::LaunchShape s = c->shape;
    // a launch that reads or writes the pinned pool itself is paced by the host link
    if (c->pool_dev != nullptr && staging >= c->pool_dev &&
        staging < c->pool_dev + uint64_t(c->n_pool_slots) * uint64_t(c->chunk_bytes))
        s.paced_groups = c->link_groups;
    const uint64_t moved = uint64_t(n_chunks) * view.by_n_lp.d * c->kg.plane_bytes;
    const uint64_t n_tokens = uint64_t(n_chunks) * c->kg.chunk_tokens;
    const bool ordered = !gather && s.paced_groups == 0 && use_ordered_scatter(c, view, n_tokens);
    if (ordered) {
        const lmc_status_t rc = prepare_order_scratch(c, n_tokens, stream);
        if (rc != LMC_OK) {
            if (e0 != nullptr) {
                c->free_time_events.push_back(e0);
                c->free_time_events.push_back(e1);
            }
            return rc;
        }
    }
    hipError_t e =
        injected_failure(c) ? hipErrorUnknown
        : gather  ? lmc::launch_gather(c->kg, view, s, ptrs, slots, n_chunks, staging, c->bad_flag_dev, stream, e0, e1)
        : ordered ? lmc::launch_scatter_ordered(c->kg, view, s, ptrs, slots, uint32_t(n_tokens), c->order, staging,
                                                c->bad_flag_dev, stream, e0, e1)
                  : lmc::launch_scatter(c->kg, view, s, ptrs, slots, n_chunks, staging, c->bad_flag_dev, stream, e0, e1);
    if (ordered && e == hipSuccess) e = hipEventRecord(c->order_free, stream);
    if (e != hipSuccess) {
        if (e0 != nullptr) {
            c->free_time_events.push_back(e0);
            c->free_time_events.push_back(e1);
        }
        HIPCHK(c, e);
    }
    if (gather) {
        c->stats.gather_launches++;
        c->stats.bytes_gathered += moved;
    } else {
        c->stats.scatter_launches++;
        c->stats.bytes_scattered += moved;
    }
    if (e0 != nullptr)
        c->timings.push_back(Timing{e0, e1, gather ? LMC_STAGE_GATHER : LMC_STAGE_SCATTER, c->cur_ticket, int32_t(n_chunks), moved});
    return LMC_OK;
}

// Copies `width` bytes per chunk between staging (chunks `stride` bytes apart) and the
// pool (offset `pool_off` inside each slot), one transfer per run of consecutive pool
// slots: a plain copy when the extents are back to back on both sides (whole chunks),
// else a rectangle copy whose rows are the chunks (layer-wise mode).  With a second
// stream the runs go to the two streams in turn; *used_second says whether any did.
static lmc_status_t copy_group(lmc_ctx *c, bool to_host, uint8_t *staging, uint64_t stride,
                        const int64_t *pool_slots, int64_t k, uint64_t pool_off, uint64_t width,
                        hipStream_t first, hipStream_t second = nullptr, bool *used_second = nullptr) {
    const uint64_t cb = uint64_t(c->chunk_bytes);
    const hipMemcpyKind kind = to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice;
    if (used_second) *used_second = false;
    // Many small pieces (a fragmented pool in layer-wise mode: one piece per chunk and step,
    // 1 MiB for one Llama layer): the runtime pays a fixed price per copy that a piece this
    // small does not cover (stores of 1 MiB pieces ran at 27-36 GB/s), so all pieces of the
    // group go in one launch of the library's copy kernel, which is told the slots.
    if (c->pool_dev != nullptr && k > 1 && width <= c->pieces_by_kernel_below &&
        ((width | stride | cb | pool_off | reinterpret_cast<uintptr_t>(staging)) % 16) == 0 &&
        c->n_pool_slots <= int64_t(INT32_MAX)) {
        int64_t runs = 1;
        for (int64_t j = 1; j < k; j++) runs += pool_slots[j] != pool_slots[j - 1] + 1;
        if (uint64_t(k) * width <= uint64_t(runs) * c->pieces_by_kernel_below && runs > 1) {
            const uint32_t groups = c->link_groups ? c->link_groups : 64u;
            for (int64_t j = 0; j < k; j += lmc::kMaxPieces) {
                const int64_t m = std::min<int64_t>(lmc::kMaxPieces, k - j);
                lmc::PieceSlots table;
                for (int64_t i = 0; i < m; i++) table.slot[i] = int32_t(pool_slots[j + i]);
                HIPCHK(c, lmc::launch_copy_pieces(c->pool_dev + pool_off, cb, staging + uint64_t(j) * stride, stride,
                                                  width, table, uint32_t(m), to_host, groups, first));
            }
            if (to_host) c->stats.bytes_d2h += uint64_t(k) * width;
            else c->stats.bytes_h2d += uint64_t(k) * width;
            return LMC_OK;
        }
    }
    bool watched = false;
    int64_t run = 0;
    for (int64_t j = 0; j < k; run++) {
        int64_t m = 1;
        while (j + m < k && pool_slots[j + m] == pool_slots[j] + m) m++;
        hipStream_t stream = first;
        const bool wanted = ((c->copy_kernel >> (to_host ? 0 : 1)) & 1u) != 0 ||
                            (to_host && c->d2h_guard_on && c->d2h_guard.use_kernel(seconds_now(c)));
        const bool by_kernel = wanted && c->pool_dev != nullptr &&
                               ((width | stride | cb | pool_off | reinterpret_cast<uintptr_t>(staging)) % 16) == 0;
        if (by_kernel) {
            // launches follow each other without a gap: one stream is enough
            uint8_t *pool_at = c->pool_dev + uint64_t(pool_slots[j]) * cb + pool_off;
            uint8_t *stage_at = staging + uint64_t(j) * stride;
            const uint32_t groups = c->link_groups ? c->link_groups : 64u;
            if (to_host) HIPCHK(c, lmc::launch_copy_rect(pool_at, cb, stage_at, stride, width, uint64_t(m), groups, stream));
            else HIPCHK(c, lmc::launch_copy_rect(stage_at, stride, pool_at, cb, width, uint64_t(m), groups, stream));
            if (to_host) c->stats.bytes_d2h += uint64_t(m) * width;
            else c->stats.bytes_h2d += uint64_t(m) * width;
            j += m;
            continue;
        }
        if (second != nullptr && (run & 1)) {
            stream = second;
            if (used_second) *used_second = true;
        }
        uint8_t *host = c->pool + uint64_t(pool_slots[j]) * cb + pool_off;
        uint8_t *dev = staging + uint64_t(j) * stride;
        // one large copy to the host per group is timed for the guard (two markers around
        // milliseconds of copy; one per group, so that a group of many copies keeps its pace)
        CopyTiming watch{nullptr, nullptr, uint64_t(m) * width};
        if (to_host && c->d2h_guard_on && !watched && watch.bytes >= lmc::CopyEngineGuard::kMinBytes &&
            get_event(c, true, &watch.start) == LMC_OK) {
            if (get_event(c, true, &watch.stop) != LMC_OK) {
                c->free_time_events.push_back(watch.start);
                watch.start = nullptr;
            } else {
                HIPCHK(c, hipEventRecord(watch.start, stream));
            }
        }
        if (m == 1 || (width == cb && stride == cb)) {
            if (to_host) HIPCHK(c, hipMemcpyAsync(host, dev, size_t(uint64_t(m) * width), kind, stream));
            else HIPCHK(c, hipMemcpyAsync(dev, host, size_t(uint64_t(m) * width), kind, stream));
        } else {
            hipError_t e = to_host ? hipMemcpy2DAsync(host, cb, dev, stride, width, size_t(m), kind, stream)
                                   : hipMemcpy2DAsync(dev, stride, host, cb, width, size_t(m), kind, stream);
            if (e == hipErrorInvalidPitchValue || e == hipErrorInvalidValue) {
                // a pitch the runtime does not take: one plain copy per chunk instead
                (void)hipGetLastError();
                for (int64_t i = 0; i < m; i++) {
                    if (to_host) HIPCHK(c, hipMemcpyAsync(host + uint64_t(i) * cb, dev + uint64_t(i) * stride, size_t(width), kind, stream));
                    else HIPCHK(c, hipMemcpyAsync(dev + uint64_t(i) * stride, host + uint64_t(i) * cb, size_t(width), kind, stream));
                }
            } else {
                HIPCHK(c, e);
            }
        }
        if (watch.start != nullptr) {
            HIPCHK(c, hipEventRecord(watch.stop, stream));
            c->copy_timings.push_back(watch);
            watched = true;
        }
        if (to_host) c->stats.bytes_d2h += uint64_t(m) * width;
        else c->stats.bytes_h2d += uint64_t(m) * width;
        j += m;
    }
    return LMC_OK;
}

// True if the pool slots are not one run of consecutive numbers (more than one transfer).
static bool several_runs(const int64_t *pool_slots, int64_t k) {
    for (int64_t j = 1; j < k; j++)
        if (pool_slots[j] != pool_slots[j - 1] + 1) return true;
    return false;
}

// Registers the operation: from here on reap() gives back what it holds.  On an error
// nothing has been registered and `op` is still the caller's.
static lmc_status_t finish_op(lmc_ctx *c, Op &&op, hipStream_t last_stream, bool enqueued,
                       uint64_t *ticket_out) {
    if (enqueued) {
        lmc_status_t rc = get_event(c, false, &op.done);
        if (rc != LMC_OK) return rc;
        const hipError_t e = injected_failure(c) ? hipErrorUnknown : hipEventRecord(op.done, last_stream);
        if (e != hipSuccess) {
            c->free_sync_events.push_back(op.done);
            op.done = nullptr;
            HIPCHK(c, e);
        }
        op.final_stream = last_stream;
    }
    if (ticket_out) *ticket_out = op.ticket;
    c->ops.push_back(std::move(op));
    return LMC_OK;
}

// Switch the ring to slots of slot_bytes.  When the size changes, the producer stream
// first waits for everything the consumer stream has been given, so no slot of the old
// division is still being read when the new division is written.
static lmc_status_t ring_reslot(lmc_ctx *c, Ring &r, uint64_t slot_bytes, hipStream_t producer,
                         hipStream_t consumer, hipStream_t producer2 = nullptr, hipStream_t consumer2 = nullptr) {
    if (slot_bytes == r.slot_bytes) return LMC_OK;
    if (r.slot_bytes != 0) {
        lmc_status_t rc = order_after(c, producer, consumer);
        if (rc == LMC_OK && producer2 != nullptr) rc = order_after(c, producer2, consumer);
        if (rc == LMC_OK && consumer2 != nullptr) rc = order_after(c, producer, consumer2);
        if (rc != LMC_OK) return rc;
    }
    // the new division takes effect only when its events exist: a failure on the way
    // leaves the ring as it was
    const uint32_t per_buf = uint32_t(std::max<uint64_t>(1, std::min<uint64_t>(r.buf_bytes / slot_bytes, 32)));
    const size_t total = r.buf.size() * per_buf;
    while (r.filled.size() < total || r.drained.size() < total) {
        std::vector<hipEvent_t> &v = r.filled.size() < total ? r.filled : r.drained;
        hipEvent_t e;
        lmc_status_t rc = get_event(c, false, &e);
        if (rc != LMC_OK) return rc;
        v.push_back(e);
    }
    r.slot_bytes = slot_bytes;
    r.slots_per_buf = per_buf;
    r.used.assign(total, 0);
    r.pos = 0;
    return LMC_OK;
}

// Next slot in turn: its index (for the events) and its address.
static size_t ring_next(Ring &r, uint8_t **ptr) {
    const size_t total = r.buf.size() * r.slots_per_buf;
    const size_t idx = size_t(r.pos++ % total);
    *ptr = r.buf[idx / r.slots_per_buf] + uint64_t(idx % r.slots_per_buf) * r.slot_bytes;
    return idx;
}

// Layer-wise mode: how many chunks' share of `view` one group (one slot, one launch) takes.
static int64_t layer_group_chunks(const lmc_ctx *c, const Ring &r, const lmc::LaunchView &view, int64_t n_chunks) {
    const int64_t fit = int64_t(r.buf_bytes / view.chunk_stride);
    return std::max<int64_t>(1, std::min({n_chunks, fit, int64_t(lmc::max_chunks_per_launch(c->kg, view))}));
}

// A chunk whose store is still on its way to the pool must be loaded after that store:
// the loading stream waits for the event behind the copies of the store's group that holds
// the chunk (a staged bulk store records one per group, so that a retrieve issued right
// behind a store of the same chunks follows it group by group, both directions of the
// link at work), or else for the store's last event (stores end on different streams, the
// D2H stream or, without staging, the gather stream, so the newest alone says nothing
// about the others).  A layer-wise store that has not been submitted completely cannot
// be waited for on the device: LMC_ERR_BUSY.
static lmc_status_t after_stores(lmc_ctx *c, const int64_t *pool_slots, int64_t n, hipStream_t waiter) {
    std::vector<hipEvent_t> events;
    for (int64_t i = 0; i < n; i++) {
        const lmc::SlotMeta &m = c->index.meta(pool_slots[i]);
        if (m.ready_ticket == 0) continue;
        const Op *o = find_op(c, m.ready_ticket);
        if (o == nullptr) continue;  // finished
        if (o->pending) return LMC_ERR_BUSY;
        hipEvent_t e = m.ready_event != nullptr ? static_cast<hipEvent_t>(m.ready_event) : o->done;
        if (e != nullptr && std::find(events.begin(), events.end(), e) == events.end()) events.push_back(e);
    }
    for (hipEvent_t e : events) HIPCHK(c, hipStreamWaitEvent(waiter, e, 0));
    return LMC_OK;
}

// Retrieve, bulk (layers_per_step == 0) or layer by layer (paper section 5.2).
static lmc_status_t do_retrieve(lmc_ctx *c, const uint64_t *ids, int64_t n_chunks,
                         const int64_t *slot_mapping, void *const *kv_layers, void *user_stream,
                         int32_t layers_per_step, uint64_t *ticket_out) {
    if (!c->has_device) return LMC_ERR_NODEVICE;
    DeviceScope dev(c);
    reap(c);
    std::vector<int64_t> pool_slots(size_t(n_chunks), 0);
    for (int64_t i = 0; i < n_chunks; i++) {
        pool_slots[size_t(i)] = c->index.find(ids[i]);
        if (pool_slots[size_t(i)] < 0) {
            c->stats.retrieve_misses++;
            return LMC_ERR_MISS;
        }
    }
    lmc::LayerPtrs ptrs;
    lmc_status_t rc = build_layer_ptrs(c, kv_layers, &ptrs);
    if (rc != LMC_OK) return rc;
    hipStream_t user = static_cast<hipStream_t>(user_stream);
    const lmc_kv_geom_t &geom = c->cfg.geom;
    const int64_t CT = geom.chunk_tokens;
    // the pages may still be in use, and the slot mapping still be on its way, by work
    // already on the caller's stream
    if (n_chunks > 0 && (rc = order_after_caller(c, c->s_scatter, user)) != LMC_OK) return rc;
    rc = validate_slots(c, slot_mapping, n_chunks * CT, c->s_scatter);
    if (rc != LMC_OK) return rc;

    const bool direct = (c->cfg.flags & LMC_FLAG_DIRECT) != 0 ||
                        (layers_per_step == 0 && n_chunks * c->chunk_bytes <= c->direct_retrieve_below);
    // without staging the scatter stream waits for every store at once; with staging each
    // group's copies wait for the stores of their own chunks (load_group)
    if ((rc = after_stores(c, pool_slots.data(), direct ? n_chunks : 0, c->s_scatter)) != LMC_OK) return rc;
    for (int64_t s : pool_slots) {
        const uint64_t t = c->index.meta(s).ready_ticket;
        const Op *o = t != 0 ? find_op(c, t) : nullptr;
        if (o != nullptr && o->pending) return LMC_ERR_BUSY;    // before anything is enqueued
    }
    begin_use(c, ids, n_chunks);   // a retrieve that is served is a use of its chunks
    end_use(c, ids, n_chunks);
    Op op;
    op.ticket = c->next_ticket++;
    c->cur_ticket = op.ticket;
    op.layerwise = layers_per_step > 0;
    if (n_chunks == 0) return finish_op(c, std::move(op), nullptr, false, ticket_out);

    Ring &ring = c->load_ring;
    const uint64_t cb = uint64_t(c->chunk_bytes);
    const int64_t per = c->cfg.staging_chunks;
    // without staging (LMC_FLAG_DIRECT, or a small bulk call): no copy, the scatter kernel
    // reads the pinned pool over the link; one launch per run of consecutive pool slots
    // (and per layer step)
    auto load_direct = [&](lmc::LaunchView view, uint64_t pool_off) -> lmc_status_t {
        view.chunk_stride = cb;  // chunks lie one pool slot apart
        const int64_t max_k = int64_t(lmc::max_chunks_per_launch(c->kg, view));
        for (int64_t i0 = 0; i0 < n_chunks;) {
            int64_t k = 1;
            while (k < max_k && i0 + k < n_chunks && pool_slots[size_t(i0 + k)] == pool_slots[size_t(i0)] + k) k++;
            lmc_status_t r = timed_launch(c, false, view, ptrs, slot_mapping + i0 * CT, uint32_t(k),
                                          c->pool_dev + uint64_t(pool_slots[size_t(i0)]) * cb + pool_off, c->s_scatter);
            if (r != LMC_OK) return r;
            c->stats.bytes_h2d += uint64_t(k) * view.by_n_lp.d * c->kg.plane_bytes;
            if ((r = force_sync(c, c->s_scatter)) != LMC_OK) return r;
            i0 += k;
        }
        return LMC_OK;
    };
    // one group: copies into the next ring buffer on the H2D stream, scatter on the
    // scatter stream; the buffer is released when the scatter has read it
    auto load_group = [&](const lmc::LaunchView &view, uint64_t pool_off, int64_t i0, int64_t k,
                          hipStream_t copy_stream, hipStream_t second) -> lmc_status_t {
        uint8_t *buf;
        const size_t b = ring_next(ring, &buf);
        if (!several_runs(&pool_slots[size_t(i0)], k)) second = nullptr;
        lmc_status_t ra = after_stores(c, &pool_slots[size_t(i0)], k, copy_stream);
        if (ra == LMC_OK && second) ra = after_stores(c, &pool_slots[size_t(i0)], k, second);
        if (ra != LMC_OK) return ra;
        if (ring.used[b]) {
            HIPCHK(c, hipStreamWaitEvent(copy_stream, ring.drained[b], 0));
            if (second) HIPCHK(c, hipStreamWaitEvent(second, ring.drained[b], 0));
        }
        bool used_second = false;
        hipEvent_t traced = nullptr;
        lmc_status_t r = trace_begin(c, copy_stream, &traced);
        if (r != LMC_OK) return r;
        r = copy_group(c, false, buf, view.chunk_stride, &pool_slots[size_t(i0)], k,
                       pool_off, view.chunk_stride, copy_stream, second, &used_second);
        // the buffer is full when the copies of both streams are in
        if (r == LMC_OK && used_second) r = order_after(c, copy_stream, second);
        if (r != LMC_OK) {
            if (traced) c->free_time_events.push_back(traced);
            return r;
        }
        if ((r = trace_end(c, copy_stream, traced, LMC_STAGE_H2D, k, uint64_t(k) * view.by_n_lp.d * c->kg.plane_bytes)) != LMC_OK)
            return r;
        HIPCHK(c, hipEventRecord(ring.filled[b], copy_stream));
        if ((r = force_sync(c, copy_stream)) != LMC_OK) return r;
        HIPCHK(c, hipStreamWaitEvent(c->s_scatter, ring.filled[b], 0));
        r = timed_launch(c, false, view, ptrs, slot_mapping + i0 * CT, uint32_t(k), buf, c->s_scatter);
        if (r != LMC_OK) return r;
        if (c->cfg.flags & LMC_FLAG_POISON_STAGING)
            HIPCHK(c, lmc::launch_fill(buf, 0xA5, uint64_t(k) * view.chunk_stride, c->s_scatter));
        HIPCHK(c, hipEventRecord(ring.drained[b], c->s_scatter));
        ring.used[b] = 1;
        return force_sync(c, c->s_scatter);
    };

    const bool two_copy_streams = !other_direction_busy(c, false);
    auto enqueue = [&]() -> lmc_status_t {
        if (direct && !op.layerwise) {
            if ((rc = load_direct(lmc::bulk_view(c->kg), 0)) != LMC_OK) return rc;
        } else if (!op.layerwise) {
            const lmc::LaunchView view = lmc::bulk_view(c->kg);
            if ((rc = ring_reslot(c, ring, ring.buf_bytes, c->s_h2d, c->s_scatter, c->s_h2d2)) != LMC_OK) return rc;
            // The link is the bottleneck and every scatter but the last hides behind the next
            // copy, so the last group is a single chunk: only its scatter is exposed.
            const int64_t edge = std::min<int64_t>(c->edge_chunks, per);
            const int64_t body = (edge > 0 && n_chunks > edge) ? n_chunks - edge : n_chunks;
            for (int64_t i0 = 0, k = 0; i0 < n_chunks; i0 += k) {
                k = i0 < body ? std::min(per, body - i0) : n_chunks - i0;
                if ((rc = load_group(view, 0, i0, k, c->s_h2d, two_copy_streams ? c->s_h2d2 : nullptr)) != LMC_OK) return rc;
            }
        } else {
            // All chunks' share of a few layers at a time: one rectangle copy per run of pool
            // slots, one scatter launch, one event that says "these layers are in place".
            const int32_t L = geom.num_layers, P = geom.num_planes;
            const uint64_t layer_bytes = uint64_t(P) * c->kg.plane_bytes;
            op.layer_done.assign(size_t(L), nullptr);
            for (int32_t l0 = 0; l0 < L; l0 += layers_per_step) {
                const int32_t kk = std::min(layers_per_step, L - l0);
                const lmc::LaunchView view = lmc::layer_view(c->kg, uint32_t(P), uint32_t(l0), uint32_t(kk));
                if (direct) {
                    if ((rc = load_direct(view, uint64_t(l0) * layer_bytes)) != LMC_OK) return rc;
                } else {
                    const int64_t cap = layer_group_chunks(c, ring, view, n_chunks);
                    if ((rc = ring_reslot(c, ring, (uint64_t(cap) * view.chunk_stride + 255) / 256 * 256, c->s_h2d,
                                          c->s_scatter, c->s_h2d2)) != LMC_OK)
                        return rc;
                    // Steps alternate between two copy streams: on one stream the runtime puts
                    // an event marker between consecutive copies, which costs the link about
                    // 20 us per step; with two streams the next step's copy is already running.
                    hipStream_t cs = (two_copy_streams && ((l0 / layers_per_step) & 1)) ? c->s_h2d2 : c->s_h2d;
                    for (int64_t i0 = 0; i0 < n_chunks; i0 += cap)
                        if ((rc = load_group(view, uint64_t(l0) * layer_bytes, i0, std::min(cap, n_chunks - i0), cs, nullptr)) != LMC_OK)
                            return rc;
                }
                hipEvent_t e;
                if ((rc = get_event(c, false, &e)) != LMC_OK) return rc;
                op.owned_events.push_back(e);
                HIPCHK(c, hipEventRecord(e, c->s_scatter));
                for (int32_t l = l0; l < l0 + kk; l++) op.layer_done[size_t(l)] = e;
            }
        }
        return LMC_OK;
    };
    op.slots = pool_slots;
    const bool layerwise = op.layerwise;
    if ((rc = enqueue()) == LMC_OK) rc = finish_op(c, std::move(op), c->s_scatter, true, ticket_out);
    if (rc != LMC_OK) {
        // Part of the call may be enqueued and still read the pool slots, which nothing
        // protects (the in-flight counts belong to a registered operation): it is waited
        // for.  Pages the call was to fill are then in an unspecified state.
        for (hipStream_t s : {c->s_h2d, c->s_h2d2, c->s_scatter}) (void)hipStreamSynchronize(s);
        (void)hipGetLastError();
        for (hipEvent_t e : op.owned_events) recycle(c, e);
        return rc;
    }
    for (int64_t s : pool_slots) c->index.meta(s).inflight++;
    c->stats.chunks_retrieved += uint64_t(n_chunks);
    // bulk: the caller's stream continues when everything is in place; layer-wise: the
    // caller orders its streams per layer with lmc_wait_layer
    if (!layerwise && c->caller_waits) HIPCHK(c, hipStreamWaitEvent(user, c->ops.back().done, 0));
    return LMC_OK;
}

// Token processor of a store: which chunks are new, and where they go.  Stops at the
// first chunk that finds no room.
static bool admit_new_chunks(lmc_ctx *c, const uint64_t *ids, int64_t n_chunks, Op *op,
                             std::vector<int64_t> *new_chunk) {
    bool fits = true;
    begin_use(c, ids, n_chunks);
    for (int64_t i = 0; i < n_chunks; i++) {
        if (c->index.find(ids[i]) >= 0) {
            c->stats.chunks_skipped_dup++;
            continue;
        }
        const int64_t s = take_slot(c, ids[i]);
        if (s < 0) {
            fits = false;
            break;
        }
        lmc::SlotMeta &m = c->index.meta(s);
        m.inflight = 1;
        m.ready_ticket = op->ticket;
        m.ready_event = nullptr;
        new_chunk->push_back(i);
        op->slots.push_back(s);
    }
    end_use(c, ids, n_chunks);
    return fits;
}

// A store that failed (a HIP error) after its chunks had been admitted.  What is already
// enqueued may still write the chunks' slots, so it is waited for; then the chunks leave
// the index again and their slots are free: no id stays behind that promises bytes which
// never arrived.  (Chunks that eviction removed to make room are not brought back.)
static void abort_store(lmc_ctx *c, const std::vector<int64_t> &slots) {
    for (hipStream_t s : {c->s_gather, c->s_d2h, c->s_d2h2}) (void)hipStreamSynchronize(s);
    (void)hipGetLastError();
    for (int64_t s : slots) c->index.erase(c->index.meta(s).id);
    c->stats.chunks_stored -= std::min<uint64_t>(c->stats.chunks_stored, slots.size());
    reap(c);
}

// Gather + D2H of the new chunks' part described by `view` (all layers, or a few),
// group by group through the store ring.
static lmc_status_t store_groups(lmc_ctx *c, const lmc::LaunchView &view, uint64_t pool_off,
                                 const lmc::LayerPtrs &ptrs, const int64_t *slot_mapping,
                                 const std::vector<int64_t> &new_chunk,
                                 const std::vector<int64_t> &new_slot, int64_t cap_chunks,
                                 bool edge_group, bool direct, bool layer_step = false, bool on_second_stream = false,
                                 std::vector<hipEvent_t> *group_events = nullptr) {
    Ring &ring = c->store_ring;
    const int64_t CT = c->cfg.geom.chunk_tokens;
    if (direct) {
        // no staging, no copy: the gather kernel writes the pinned pool over the link; one
        // launch per run of chunks that are consecutive both in the slot mapping and in the pool
        lmc::LaunchView v = view;
        v.chunk_stride = uint64_t(c->chunk_bytes);
        const size_t max_k = size_t(lmc::max_chunks_per_launch(c->kg, v));
        for (size_t j0 = 0; j0 < new_chunk.size();) {
            size_t k = 1;
            while (k < max_k && j0 + k < new_chunk.size() && new_chunk[j0 + k] == new_chunk[j0] + int64_t(k) &&
                   new_slot[j0 + k] == new_slot[j0] + int64_t(k))
                k++;
            lmc_status_t rc = timed_launch(c, true, v, ptrs, slot_mapping + new_chunk[j0] * CT, uint32_t(k),
                                           c->pool_dev + uint64_t(new_slot[j0]) * v.chunk_stride + pool_off,
                                           c->s_gather);
            if (rc != LMC_OK) return rc;
            c->stats.bytes_d2h += uint64_t(k) * v.by_n_lp.d * c->kg.plane_bytes;
            if ((rc = force_sync(c, c->s_gather)) != LMC_OK) return rc;
            j0 += k;
        }
        return LMC_OK;
    }
    const size_t per = size_t(cap_chunks);
    const bool two_copy_streams = !other_direction_busy(c, true);
    hipStream_t copies = on_second_stream ? c->s_d2h2 : c->s_d2h, other = on_second_stream ? c->s_d2h : c->s_d2h2;
    for (size_t j0 = 0; j0 < new_chunk.size();) {
        // one launch covers chunks that are consecutive in the caller's slot mapping.
        // Only the first gather is exposed (later ones hide behind the previous copy),
        // so the first group is a single chunk and the link starts working at once.
        const size_t edge = edge_group ? size_t(std::min<int64_t>(c->edge_chunks, int64_t(per))) : 0;
        const size_t cap = (j0 == 0 && edge > 0 && new_chunk.size() > edge) ? edge : per;
        size_t k = 1;
        while (k < cap && j0 + k < new_chunk.size() && new_chunk[j0 + k] == new_chunk[j0] + int64_t(k)) k++;
        uint8_t *buf;
        const size_t b = ring_next(ring, &buf);
        if (ring.used[b]) HIPCHK(c, hipStreamWaitEvent(c->s_gather, ring.drained[b], 0));
        lmc_status_t rc = timed_launch(c, true, view, ptrs, slot_mapping + new_chunk[j0] * CT, uint32_t(k),
                                       buf, c->s_gather);
        if (rc != LMC_OK) return rc;
        HIPCHK(c, hipEventRecord(ring.filled[b], c->s_gather));
        if ((rc = force_sync(c, c->s_gather)) != LMC_OK) return rc;
        HIPCHK(c, hipStreamWaitEvent(copies, ring.filled[b], 0));
        // a layer-wise step has the two streams step by step, not run by run (as the steps of a retrieve)
        hipStream_t second = (two_copy_streams && !(layer_step && c->store_step_streams == 2) && several_runs(&new_slot[j0], int64_t(k)))
                                 ? other : nullptr;
        if (second) HIPCHK(c, hipStreamWaitEvent(second, ring.filled[b], 0));
        bool used_second = false;
        hipEvent_t traced = nullptr;
        if ((rc = trace_begin(c, copies, &traced)) != LMC_OK) return rc;
        rc = copy_group(c, true, buf, view.chunk_stride, &new_slot[j0], int64_t(k), pool_off,
                        view.chunk_stride, copies, second, &used_second);
        // the group's copy stream stands for the whole group: it ends after the other stream's copies
        if (rc == LMC_OK && used_second) rc = order_after(c, copies, second);
        if (rc != LMC_OK) {
            if (traced) c->free_time_events.push_back(traced);
            return rc;
        }
        if ((rc = trace_end(c, copies, traced, LMC_STAGE_D2H, int64_t(k), uint64_t(k) * view.by_n_lp.d * c->kg.plane_bytes)) != LMC_OK)
            return rc;
        if (c->cfg.flags & LMC_FLAG_POISON_STAGING)
            HIPCHK(c, lmc::launch_fill(buf, 0xA5, uint64_t(k) * view.chunk_stride, copies));
        HIPCHK(c, hipEventRecord(ring.drained[b], copies));
        ring.used[b] = 1;
        if (group_events != nullptr) {
            // "these chunks are in the pool": an event of the group's own (drained[b] is recorded
            // again whenever the buffer comes round), kept by the store until it is reaped
            hipEvent_t in_pool;
            if ((rc = get_event(c, false, &in_pool)) != LMC_OK) return rc;
            group_events->push_back(in_pool);
            HIPCHK(c, hipEventRecord(in_pool, copies));
            for (size_t j = j0; j < j0 + k; j++) c->index.meta(new_slot[j]).ready_event = in_pool;
        }
        if ((rc = force_sync(c, copies)) != LMC_OK) return rc;
        j0 += k;
    }
    return LMC_OK;
}

static lmc_status_t device_only(lmc_ctx_t *c, bool gather, void *const *kv_layers,
                                const int64_t *slot_mapping, int64_t n_chunks, uint8_t *staging,
                                void *stream) {
    if (!c || n_chunks < 0 || !kv_layers || (n_chunks > 0 && (!slot_mapping || !staging)))
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    if (reinterpret_cast<uintptr_t>(staging) % c->kg.vec) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    c->cur_ticket = 0;
    DeviceScope dev(c);
    reap(c);
    lmc::LayerPtrs ptrs;
    lmc_status_t rc = build_layer_ptrs(c, kv_layers, &ptrs);
    if (rc != LMC_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t CT = c->cfg.geom.chunk_tokens;
    if ((rc = validate_slots(c, slot_mapping, n_chunks * CT, s)) != LMC_OK) return rc;
    const lmc::LaunchView view = lmc::bulk_view(c->kg);
    const int64_t per = int64_t(lmc::max_chunks_per_launch(c->kg, view));
    for (int64_t i0 = 0; i0 < n_chunks; i0 += per) {
        const int64_t k = std::min(per, n_chunks - i0);
        rc = timed_launch(c, gather, view, ptrs, slot_mapping + i0 * CT, uint32_t(k),
                          staging + i0 * c->chunk_bytes, s);
        if (rc != LMC_OK) return rc;
    }
    return LMC_OK;
}

}  // namespace lmci

using namespace lmci;

extern "C" {

lmc_status_t lmc_store(lmc_ctx_t *c, void *const *kv_layers, const int64_t *slot_mapping,
                       const uint64_t *ids, int64_t n_chunks, void *stream_to_wait_on,
                       uint64_t *ticket_out) {
    if (!c || n_chunks < 0 || !kv_layers || (n_chunks > 0 && (!slot_mapping || !ids)))
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    reap(c);
    lmc::LayerPtrs ptrs;
    lmc_status_t rc = build_layer_ptrs(c, kv_layers, &ptrs);
    if (rc != LMC_OK) return rc;
    hipStream_t user = static_cast<hipStream_t>(stream_to_wait_on);
    const int64_t CT = c->cfg.geom.chunk_tokens;
    if (n_chunks > 0 && (rc = order_after_caller(c, c->s_gather, user)) != LMC_OK) return rc;
    if ((rc = validate_slots(c, slot_mapping, n_chunks * CT, c->s_gather)) != LMC_OK) return rc;

    Op op;
    op.ticket = c->next_ticket++;
    c->cur_ticket = op.ticket;
    std::vector<int64_t> new_chunk;
    const bool fits = admit_new_chunks(c, ids, n_chunks, &op, &new_chunk);
    c->stats.chunks_stored += new_chunk.size();
    const bool direct = (c->cfg.flags & LMC_FLAG_DIRECT) != 0 ||
                        int64_t(new_chunk.size()) * c->chunk_bytes <= c->direct_store_below;
    rc = direct ? LMC_OK : ring_reslot(c, c->store_ring, c->store_ring.buf_bytes, c->s_gather, c->s_d2h, nullptr, c->s_d2h2);
    if (rc == LMC_OK)
        rc = store_groups(c, lmc::bulk_view(c->kg), 0, ptrs, slot_mapping, new_chunk, op.slots,
                          c->cfg.staging_chunks, true, direct, false, false, &op.owned_events);
    if (rc == LMC_OK)
        rc = finish_op(c, std::move(op), direct ? c->s_gather : c->s_d2h, !new_chunk.empty(), ticket_out);
    if (rc != LMC_OK) {
        abort_store(c, op.slots);   // finish_op registers as its last step: op is still whole
        for (hipEvent_t e : op.owned_events) recycle(c, e);
        return rc;
    }
    return fits ? LMC_OK : LMC_ERR_NOMEM;
}

lmc_status_t lmc_store_begin(lmc_ctx_t *c, const int64_t *slot_mapping, const uint64_t *ids,
                             int64_t n_chunks, void *stream_to_wait_on, uint64_t *ticket_out) {
    if (!c || n_chunks < 0 || (n_chunks > 0 && (!slot_mapping || !ids))) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    reap(c);
    lmc_status_t rc;
    hipStream_t user = static_cast<hipStream_t>(stream_to_wait_on);
    const int64_t CT = c->cfg.geom.chunk_tokens;
    if (n_chunks > 0 && (rc = order_after_caller(c, c->s_gather, user)) != LMC_OK) return rc;
    if ((rc = validate_slots(c, slot_mapping, n_chunks * CT, c->s_gather)) != LMC_OK) return rc;
    Op op;
    op.ticket = c->next_ticket++;
    op.layerwise = true;
    const bool fits = admit_new_chunks(c, ids, n_chunks, &op, &op.new_chunk);
    c->stats.chunks_stored += op.new_chunk.size();
    op.pending = !op.new_chunk.empty();   // nothing new: the ticket is complete at once
    op.slot_mapping = slot_mapping;
    op.layer_done.assign(size_t(c->cfg.geom.num_layers), nullptr);
    if (ticket_out) *ticket_out = op.ticket;
    c->ops.push_back(std::move(op));
    return fits ? LMC_OK : LMC_ERR_NOMEM;
}

lmc_status_t lmc_store_layers(lmc_ctx_t *c, uint64_t ticket, int32_t first_layer, int32_t n_layers,
                              void *const *kv_layers, void *stream_to_wait_on) {
    if (!c || !kv_layers || n_layers < 1 || first_layer < 0) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    reap(c);
    const lmc_kv_geom_t &geom = c->cfg.geom;
    Op *op = find_op(c, ticket);
    if (op == nullptr) {
        // a layer-wise store with nothing new completes at once; its layers are accepted
        // and ignored so that the caller's per-layer loop needs no special case
        return (ticket != 0 && ticket < c->next_ticket && first_layer + n_layers <= geom.num_layers)
                   ? LMC_OK : LMC_ERR_INVAL;
    }
    if (!op->pending || first_layer != op->next_layer || first_layer + n_layers > geom.num_layers)
        return LMC_ERR_INVAL;
    c->cur_ticket = op->ticket;
    lmc::LayerPtrs ptrs;
    lmc_status_t rc = build_layer_ptrs(c, kv_layers, &ptrs);
    if (rc != LMC_OK) return rc;
    const lmc::LaunchView view = lmc::layer_view(c->kg, uint32_t(geom.num_planes), uint32_t(first_layer),
                                                 uint32_t(n_layers));
    const uint64_t layer_bytes = uint64_t(geom.num_planes) * c->kg.plane_bytes;
    const int64_t cap = layer_group_chunks(c, c->store_ring, view, int64_t(op->new_chunk.size()));
    const bool direct = (c->cfg.flags & LMC_FLAG_DIRECT) != 0;
    // Steps take the two copy streams in turn (as the steps of a layer-wise retrieve do):
    // between two copies of one stream the runtime leaves the link idle for some 20 us,
    // 7 % of a step of one Llama-3-8B layer, while on the other stream (another hardware
    // queue, see arrange_streams) the next step's copy is ready to start.  Not while a
    // retrieve is under way, whose kernels that stream would hold up.
    const bool on_second = !direct && (op->steps & 1) != 0 && c->store_step_streams == 2 && !other_direction_busy(c, true);
    hipStream_t last = direct ? c->s_gather : on_second ? c->s_d2h2 : c->s_d2h;
    // this layer's KV was produced by work already on the caller's stream
    rc = order_after_caller(c, c->s_gather, static_cast<hipStream_t>(stream_to_wait_on));
    if (rc == LMC_OK && !direct)
        rc = ring_reslot(c, c->store_ring, (uint64_t(cap) * view.chunk_stride + 255) / 256 * 256, c->s_gather, c->s_d2h,
                         nullptr, c->s_d2h2);
    if (rc == LMC_OK)
        rc = store_groups(c, view, uint64_t(first_layer) * layer_bytes, ptrs, op->slot_mapping, op->new_chunk,
                          op->slots, cap, false, direct, true, on_second);
    hipEvent_t e = nullptr;
    if (rc == LMC_OK) rc = get_event(c, false, &e);
    if (rc == LMC_OK) {
        op->owned_events.push_back(e);
        rc = [&]() -> lmc_status_t {
            HIPCHK(c, hipEventRecord(e, last));
            if (first_layer + n_layers == geom.num_layers) {
                // the ticket is complete when the steps of both streams are
                lmc_status_t r = (op->both_copy_streams || on_second)
                                     ? order_after(c, last, on_second ? c->s_d2h : c->s_d2h2) : LMC_OK;
                if (r == LMC_OK) r = get_event(c, false, &op->done);
                if (r != LMC_OK) return r;
                op->owned_events.push_back(op->done);   // given back with the others if the record fails
                HIPCHK(c, hipEventRecord(op->done, last));
                op->owned_events.pop_back();
                op->final_stream = last;
            }
            return LMC_OK;
        }();
    }
    if (rc != LMC_OK) {
        // the store cannot be completed any more: it is taken back as a whole
        const uint64_t t = op->ticket;
        auto it = std::find_if(c->ops.begin(), c->ops.end(), [t](const Op &o) { return o.ticket == t; });
        const Op gone = std::move(*it);
        c->ops.erase(it);
        abort_store(c, gone.slots);
        for (hipEvent_t x : gone.owned_events) recycle(c, x);
        return rc;
    }
    for (int32_t l = first_layer; l < first_layer + n_layers; l++) op->layer_done[size_t(l)] = e;
    op->next_layer = first_layer + n_layers;
    op->steps++;
    op->both_copy_streams = op->both_copy_streams || on_second;
    if (op->next_layer == geom.num_layers) op->pending = false;
    return LMC_OK;
}

lmc_status_t lmc_retrieve_layerwise(lmc_ctx_t *c, const uint64_t *ids, int64_t n_chunks,
                                    const int64_t *slot_mapping, void *const *kv_layers,
                                    int32_t layers_per_step, void *stream_to_wait_on,
                                    uint64_t *ticket_out) {
    if (!c || n_chunks < 0 || !kv_layers || layers_per_step < 1 ||
        (n_chunks > 0 && (!slot_mapping || !ids)))
        return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    return do_retrieve(c, ids, n_chunks, slot_mapping, kv_layers, stream_to_wait_on,
                       std::min(layers_per_step, c->cfg.geom.num_layers), ticket_out);
}

lmc_status_t lmc_wait_layer(lmc_ctx_t *c, uint64_t ticket, int32_t layer, void *stream) {
    if (!c || ticket == 0 || layer < 0 || layer >= c->cfg.geom.num_layers) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (ticket >= c->next_ticket) return LMC_ERR_INVAL;
    const Op *op = find_op(c, ticket);
    if (op == nullptr) return LMC_OK;                       // finished long ago
    if (!op->layerwise) return LMC_ERR_INVAL;
    if (op->layer_done.empty() || (op->layer_done[size_t(layer)] == nullptr && !op->pending))
        return LMC_OK;                                      // nothing was enqueued for it
    if (op->layer_done[size_t(layer)] == nullptr) return LMC_ERR_BUSY;  // layer not submitted yet
    HIPCHK(c, hipStreamWaitEvent(static_cast<hipStream_t>(stream), op->layer_done[size_t(layer)], 0));
    return LMC_OK;
}

lmc_status_t lmc_retrieve(lmc_ctx_t *c, const uint64_t *ids, int64_t n_chunks,
                          const int64_t *slot_mapping, void *const *kv_layers,
                          void *stream_to_signal, uint64_t *ticket_out) {
    if (!c || n_chunks < 0 || !kv_layers || (n_chunks > 0 && (!slot_mapping || !ids)))
        return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    return do_retrieve(c, ids, n_chunks, slot_mapping, kv_layers, stream_to_signal, 0, ticket_out);
}

lmc_status_t lmc_retrieve_batch(lmc_ctx_t *c, int64_t n_req, const int64_t *off,
                                const uint64_t *ids, const int64_t *slot_mapping,
                                void *const *kv_layers, void *stream_to_signal,
                                uint64_t *ticket_out) {
    if (!c || n_req < 0 || !off || !kv_layers || off[0] != 0) return LMC_ERR_INVAL;
    for (int64_t r = 0; r < n_req; r++)
        if (off[r + 1] < off[r]) return LMC_ERR_INVAL;
    const int64_t total = off[n_req];
    if (total > 0 && (!ids || !slot_mapping)) return LMC_ERR_INVAL;
    // The requests' chunks and slot mappings are already back to back, so the batch is
    // one stream of chunks: kernel launches and copies run across request borders.
    std::lock_guard<std::mutex> lock(c->mu);
    return do_retrieve(c, ids, total, slot_mapping, kv_layers, stream_to_signal, 0, ticket_out);
}

lmc_status_t lmc_gather(lmc_ctx_t *c, void *const *kv_layers, const int64_t *slot_mapping,
                        int64_t n_chunks, void *staging_dev, void *stream) {
    return device_only(c, true, kv_layers, slot_mapping, n_chunks, static_cast<uint8_t *>(staging_dev), stream);
}

lmc_status_t lmc_scatter(lmc_ctx_t *c, const void *staging_dev, const int64_t *slot_mapping,
                         int64_t n_chunks, void *const *kv_layers, void *stream) {
    return device_only(c, false, kv_layers, slot_mapping, n_chunks,
                       static_cast<uint8_t *>(const_cast<void *>(staging_dev)), stream);
}

}  // extern "C"
