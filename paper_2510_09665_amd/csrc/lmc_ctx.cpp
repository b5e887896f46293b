// liblmc context, pipelines and C ABI (see include/lmc.h for the contract).
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
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/lmc.h"
#include "lmc_guard.hpp"
#include "lmc_index.hpp"
#include "lmc_kernels.hpp"

// Device memory for the one entry point that must not allocate (lmc_store_static): the
// staging buffer of that call.  Every GPU the library's code is loaded on holds its own
// copy of this array, at its own address, until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; the address that kernels and copies
// use is the one looked up per device in static_scratch_at.
static __device__ __align__(256) uint8_t scratch[LMC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
uint8_t *static_scratch_at[kMaxDevices];   // per device ordinal; null = not looked up yet
std::mutex static_scratch_mu;

// Looks up, once per device and with that device current, where this GPU keeps `scratch`.
hipError_t resolve_static_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return hipSuccess;   // lmc_store_static refuses such a device
    std::lock_guard<std::mutex> lock(static_scratch_mu);
    if (static_scratch_at[device] != nullptr) return hipSuccess;
    void *at = nullptr;
    const hipError_t e = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (at == nullptr) return hipErrorInvalidSymbol;
    static_scratch_at[device] = static_cast<uint8_t *>(at);
    return hipSuccess;
}

uint8_t *static_scratch_of(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(static_scratch_mu);
    return static_scratch_at[device];
}

// Staging ring of one direction.  The memory is num_staging allocations of buf_bytes;
// it is handed out in slots of slot_bytes (bulk mode: one slot per allocation;
// layer-wise mode: many small slots, so that a call seldom has to wait for a slot).
// Each slot has a `filled` event (producer done) and a `drained` event (consumer done).
struct Ring {
    std::vector<uint8_t *> buf;
    uint64_t buf_bytes = 0, slot_bytes = 0;
    uint32_t slots_per_buf = 1;
    std::vector<hipEvent_t> filled, drained;
    std::vector<char> used;
    uint64_t pos = 0;
};

struct Op {
    uint64_t ticket = 0;
    hipEvent_t done = nullptr;       // null: nothing enqueued (yet) for this ticket
    hipStream_t final_stream = nullptr;  // the library stream `done` was recorded on
    std::vector<int64_t> slots;      // pool slots whose in-flight count this op holds
    // layer-wise operations (paper section 5.2)
    bool layerwise = false;
    bool pending = false;                 // a store whose layers have not all been submitted
    int32_t next_layer = 0;               // first layer not yet submitted
    int32_t steps = 0;                    // pending store: lmc_store_layers calls served so far
    bool both_copy_streams = false;       // pending store: steps went to the two copy streams in turn
    std::vector<int64_t> new_chunk;       // pending store: chunk numbers that are new
    const int64_t *slot_mapping = nullptr;  // pending store: the caller's slot mapping
    std::vector<hipEvent_t> layer_done;   // per layer: event after which the layer is in place
    std::vector<hipEvent_t> owned_events; // the distinct events behind layer_done
};

struct Timing {
    hipEvent_t start, stop;
    bool is_gather;
};

struct CopyTiming {   // a large device-to-host copy by the runtime, watched by the guard
    hipEvent_t start, stop;
    uint64_t bytes;
};

}  // namespace

struct lmc_ctx {
    lmc_config_t cfg{};
    lmc::KernelGeom kg{};
    lmc::LaunchShape shape{};
    uint32_t link_groups = 64;  // workgroups of a launch whose other side is the pinned pool; 0 = as for HBM
    // Which copies between staging and the pool the library's own link-paced copy kernel
    // makes instead of hipMemcpyAsync: bit 0 = to the host, bit 1 = from the host.  Off
    // by default: the runtime's copies are 2-3 % faster.  But for some seconds after tens
    // of GiB of device or pinned memory have been freed or allocated in the process, the
    // runtime's device-to-host copies inside a store ran at 31.5 GB/s instead of 57 on
    // the machine this was measured on (not with HSA_ENABLE_SDMA=0, which points at the
    // copy engines being busy with the driver's own work on that memory); the kernel's
    // 55 GB/s does not depend on that.
    uint32_t copy_kernel = 0;
    // ... and the guard that switches device-to-host copies to the kernel by itself while
    // the runtime's are slow (lmc_guard.hpp).  Off unless asked for (lmc_tune "d2h_guard").
    // Measured on a 10 GiB request: in a fresh process's first seconds the guard lifts the
    // path from 44.5 to 54.5 GB/s; later, after a context with a large pool has been created,
    // it holds the copies on the copy kernel (55.7 GB/s) for seconds although the runtime's
    // were back at 56.8 after one store.  Steady state is the same either way.
    bool d2h_guard_on = false;
    uint64_t pieces_by_kernel_below = uint64_t(2) << 20;   // bytes per transfer; see copy_group
    int32_t store_step_streams = 2;   // copy streams the steps of a layer-wise store take in turn
    bool caller_waits = true;     // a bulk retrieve ends with the caller's stream waiting for it
    lmc::CopyEngineGuard d2h_guard;
    std::vector<CopyTiming> copy_timings;
    std::chrono::steady_clock::time_point born = std::chrono::steady_clock::now();
    int64_t edge_chunks = 1;  // size of the group at the exposed end of a pipeline; 0 = no special group
    // Scatter launches in the order of the destination (lmc_kernels.hpp): 0 = never, 1 = when
    // the launch fills enough pages per plane for neighbours to exist (ordered_min_pages pages
    // and at least one block in ordered_min_density_inv of the plane), 2 = whenever possible.
    // Off: measured on MI355X it loses to the plain order at every density tried (2048 of
    // 8192, 6480 of 16384, 4096 of 8192 blocks per plane: 2-6 % slower), because the jumps it
    // takes off the writes land on the reads of the staging buffer.  Kept as a switch so that
    // the benchmark can show the comparison.
    int32_t scatter_order = 0;
    int64_t ordered_min_pages = 1024, ordered_min_density_inv = 8;
    lmc::OrderScratch order{};         // device scratch of such launches, grown on demand
    uint64_t order_cap_tokens = 0;
    hipEvent_t order_free = nullptr;   // the last such launch has finished with the scratch
    std::vector<void *> order_retired; // outgrown scratch, freed with the context
    uint64_t use_calls = 0;         // number of the latest call that used chunks (recency of use)
    std::vector<uint64_t> evicted;  // LMC_FLAG_EVICT_LRU: ids evicted and not yet drained
    // Bulk calls that move at most this many bytes skip staging and the copy engine (the
    // kernel itself crosses the link).  Small transfers are bound by launch latencies, which
    // one launch instead of kernel, event, copy, event halves; up to 64 MiB the single
    // launch is still 2-5 % faster and is over within a millisecond or so, beyond that
    // the staged pipeline keeps the compute units free.  0 = never.
    int64_t direct_store_below = int64_t(64) << 20;
    int64_t direct_retrieve_below = int64_t(64) << 20;
    int64_t chunk_bytes = 0;
    int64_t n_pool_slots = 0;
    uint8_t *pool = nullptr;
    uint8_t *pool_dev = nullptr;   // the pool's address as the GPU sees it (LMC_FLAG_DIRECT)
    bool has_device = false;
    lmc::ChunkIndex index;
    std::mutex mu;
    hipStream_t s_gather = nullptr, s_d2h = nullptr, s_h2d = nullptr, s_scatter = nullptr;
    // second copy streams: where consecutive transfers cannot be merged into one (layer
    // steps, scattered pool slots) they alternate between the two streams of their
    // direction, because back-to-back copies on one stream leave the link idle in between
    hipStream_t s_h2d2 = nullptr, s_d2h2 = nullptr;
    std::vector<hipStream_t> retired_streams;   // see arrange_streams; destroyed with the context, after the events
    Ring store_ring, load_ring;
    int32_t *bad_flag_host = nullptr, *bad_flag_dev = nullptr;
    std::deque<Op> ops;
    std::deque<Timing> timings;
    uint64_t next_ticket = 1;
    std::vector<hipEvent_t> free_sync_events, free_time_events, all_events;
    // Threads that sleep in hipEventSynchronize with the mutex released.  While there are
    // any, events that become free are parked in held_events instead of going back to the
    // free list: an event somebody sleeps on is then never recorded anew under them.
    int waiters = 0;
    std::vector<hipEvent_t> held_events;
    // Test hook (lmc_tune "fail_hip_after"): the n-th checked HIP call from now is not made
    // and counts as failed.  Forces the error paths without any fault on the device.
    uint32_t fail_hip_after = 0;
    lmc_stats_t stats{};
    int32_t last_hip_error = 0;
};

namespace {

// A failed HIP call is reported through the library's own status and
// lmc_last_hip_error(); the runtime's per-thread "last error" is cleared so that it does
// not surface in the caller's next, unrelated HIP call.
inline bool injected_failure(lmc_ctx *c) {
    return c->fail_hip_after > 0 && --c->fail_hip_after == 0;
}

#define HIPCHK(ctx, expr)                                  \
    do {                                                   \
        hipError_t e_ = injected_failure(ctx) ? hipErrorUnknown : (expr); \
        if (e_ != hipSuccess) {                            \
            (ctx)->last_hip_error = int32_t(e_);           \
            (void)hipGetLastError();                       \
            return LMC_ERR_HIP;                            \
        }                                                  \
    } while (0)

// Makes the context's device current for the scope of one API call.
class DeviceScope {
public:
    explicit DeviceScope(const lmc_ctx *c) {
        if (c->has_device && hipGetDevice(&prev_) == hipSuccess && prev_ != c->cfg.device) {
            if (hipSetDevice(c->cfg.device) == hipSuccess) restore_ = true;
        }
    }
    ~DeviceScope() {
        if (restore_) (void)hipSetDevice(prev_);
    }

private:
    int prev_ = 0;
    bool restore_ = false;
};

// The mapped flag block holds 16 words: word 0 is set by the gather / scatter kernels on a
// slot outside the pages, word kCheckWord by the check kernel of LMC_FLAG_VALIDATE_SLOTS.
constexpr int kCheckWord = 8;

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

int64_t gcd_pow2(int64_t a, int64_t cap) {
    int64_t v = cap;
    while (v > 1 && (a % v) != 0) v >>= 1;
    return v;
}

// Fill KernelGeom from the public geometry; LMC_ERR_INVAL if it cannot be expressed.
lmc_status_t derive_geometry(const lmc_kv_geom_t &g, lmc::KernelGeom *k, int64_t *chunk_bytes) {
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
            if (m.ready_ticket == op.ticket) m.ready_ticket = 0;
        }
        c->ops.erase(c->ops.begin() + long(i));
    }
    for (size_t i = 0; i < c->timings.size();) {
        Timing &t = c->timings[i];
        if (hipEventQuery(t.stop) == hipSuccess) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
                if (t.is_gather) {
                    c->stats.gather_ms += ms;
                    c->stats.timed_gather_launches++;
                } else {
                    c->stats.scatter_ms += ms;
                    c->stats.timed_scatter_launches++;
                }
            }
            c->free_time_events.push_back(t.start);
            c->free_time_events.push_back(t.stop);
            c->timings.erase(c->timings.begin() + long(i));
        } else {
            i++;
        }
    }
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
// when the store's last gather has run).
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

// Does this scatter launch go in the order of the destination?  It pays when the launch
// finds neighbours among its pages: many pages per plane, and a fair share of the plane.
bool use_ordered_scatter(const lmc_ctx *c, const lmc::LaunchView &view, uint64_t n_tokens) {
    if (c->scatter_order == 0 || !lmc::ordered_scatter_fits(c->kg, view, c->shape, n_tokens)) return false;
    if (c->scatter_order >= 2) return true;
    const int64_t pages = int64_t(n_tokens) / c->cfg.geom.block_size;
    return pages >= c->ordered_min_pages && pages * c->ordered_min_density_inv >= int64_t(c->cfg.geom.num_blocks);
}

// The scratch of an ordered launch: allocated when first needed, grown when a launch has
// more tokens than any before (the outgrown arrays may still be in use by a launch under
// way and are kept until the context goes).  `stream` is made to wait for the previous
// ordered launch, which may have run on another stream: one set serves one launch at a time.
lmc_status_t prepare_order_scratch(lmc_ctx *c, uint64_t n_tokens, hipStream_t stream) {
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
    if (c->cfg.flags & LMC_FLAG_TIMING) {
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
    if (e0 != nullptr) c->timings.push_back(Timing{e0, e1, gather});
    return LMC_OK;
}

lmc_status_t force_sync(lmc_ctx *c, hipStream_t s) {
    if (c->cfg.flags & LMC_FLAG_FORCE_SYNC) HIPCHK(c, hipStreamSynchronize(s));
    return LMC_OK;
}

// Copies `width` bytes per chunk between staging (chunks `stride` bytes apart) and the
// pool (offset `pool_off` inside each slot), one transfer per run of consecutive pool
// slots: a plain copy when the extents are back to back on both sides (whole chunks),
// else a rectangle copy whose rows are the chunks (layer-wise mode).  With a second
// stream the runs go to the two streams in turn; *used_second says whether any did.
lmc_status_t copy_group(lmc_ctx *c, bool to_host, uint8_t *staging, uint64_t stride,
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
bool several_runs(const int64_t *pool_slots, int64_t k) {
    for (int64_t j = 1; j < k; j++)
        if (pool_slots[j] != pool_slots[j - 1] + 1) return true;
    return false;
}

// Registers the operation: from here on reap() gives back what it holds.  On an error
// nothing has been registered and `op` is still the caller's.
lmc_status_t finish_op(lmc_ctx *c, Op &&op, hipStream_t last_stream, bool enqueued,
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

// Switch the ring to slots of slot_bytes.  When the size changes, the producer stream
// first waits for everything the consumer stream has been given, so no slot of the old
// division is still being read when the new division is written.
lmc_status_t ring_reslot(lmc_ctx *c, Ring &r, uint64_t slot_bytes, hipStream_t producer,
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
size_t ring_next(Ring &r, uint8_t **ptr) {
    const size_t total = r.buf.size() * r.slots_per_buf;
    const size_t idx = size_t(r.pos++ % total);
    *ptr = r.buf[idx / r.slots_per_buf] + uint64_t(idx % r.slots_per_buf) * r.slot_bytes;
    return idx;
}

// Layer-wise mode: how many chunks' share of `view` one group (one slot, one launch) takes.
int64_t layer_group_chunks(const lmc_ctx *c, const Ring &r, const lmc::LaunchView &view, int64_t n_chunks) {
    const int64_t fit = int64_t(r.buf_bytes / view.chunk_stride);
    return std::max<int64_t>(1, std::min({n_chunks, fit, int64_t(lmc::max_chunks_per_launch(c->kg, view))}));
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
lmc_status_t sync_unlocked(lmc_ctx *c, std::unique_lock<std::mutex> &lock,
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

// The store that fills the slot of chunk `id`, if it is still under way: its `done`
// event goes to *ev (null = nothing to wait for).  LMC_ERR_MISS / LMC_ERR_BUSY as lmc_get_host.
lmc_status_t pending_fill(lmc_ctx *c, uint64_t id, int64_t *slot_out, hipEvent_t *ev) {
    *ev = nullptr;
    const int64_t s = c->index.find(id);
    if (s < 0) return LMC_ERR_MISS;
    *slot_out = s;
    const uint64_t store_ticket = c->index.meta(s).ready_ticket;
    if (store_ticket != 0) {
        const Op *o = find_op(c, store_ticket);
        if (o != nullptr && o->pending) return LMC_ERR_BUSY;
        if (o != nullptr) *ev = o->done;
    }
    return LMC_OK;
}

// A chunk whose store is still on its way to the pool must be loaded after that store:
// the loading stream waits for every such store (stores end on different streams, the
// D2H stream or, without staging, the gather stream, so the newest alone says nothing
// about the others).  A layer-wise store that has not been submitted completely cannot
// be waited for on the device: LMC_ERR_BUSY.
lmc_status_t after_stores(lmc_ctx *c, const std::vector<int64_t> &pool_slots, hipStream_t waiter) {
    std::vector<uint64_t> tickets;
    for (int64_t s : pool_slots) {
        const uint64_t t = c->index.meta(s).ready_ticket;
        if (t == 0 || (!tickets.empty() && tickets.back() == t)) continue;
        const Op *o = find_op(c, t);
        if (o == nullptr) continue;  // finished
        if (o->pending) return LMC_ERR_BUSY;
        if (std::find(tickets.begin(), tickets.end(), t) == tickets.end()) tickets.push_back(t);
    }
    for (uint64_t t : tickets) {
        const Op *o = find_op(c, t);
        if (o != nullptr && o->done != nullptr) HIPCHK(c, hipStreamWaitEvent(waiter, o->done, 0));
    }
    return LMC_OK;
}

// Retrieve, bulk (layers_per_step == 0) or layer by layer (paper section 5.2).
lmc_status_t do_retrieve(lmc_ctx *c, const uint64_t *ids, int64_t n_chunks,
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
    if ((rc = after_stores(c, pool_slots, direct ? c->s_scatter : c->s_h2d)) != LMC_OK) return rc;
    if (!direct && (rc = after_stores(c, pool_slots, c->s_h2d2)) != LMC_OK) return rc;
    begin_use(c, ids, n_chunks);   // a retrieve that is served is a use of its chunks
    end_use(c, ids, n_chunks);
    Op op;
    op.ticket = c->next_ticket++;
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
        if (ring.used[b]) {
            HIPCHK(c, hipStreamWaitEvent(copy_stream, ring.drained[b], 0));
            if (second) HIPCHK(c, hipStreamWaitEvent(second, ring.drained[b], 0));
        }
        bool used_second = false;
        lmc_status_t r = copy_group(c, false, buf, view.chunk_stride, &pool_slots[size_t(i0)], k,
                                    pool_off, view.chunk_stride, copy_stream, second, &used_second);
        if (r != LMC_OK) return r;
        // the buffer is full when the copies of both streams are in
        if (used_second && (r = order_after(c, copy_stream, second)) != LMC_OK) return r;
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

// Does work on stream `other` stand still while a copy runs on `busy`?  HIP maps streams
// onto a few hardware queues and a queue runs its entries in order, so two streams of one
// queue do not overlap.  A copy of `nbytes` that only reads the pool is enqueued on `busy`
// (with by_kernel: the link-paced copy kernel, what direct mode runs on the kernel streams)
// and right behind it, on `other`, a small kernel that depends on nothing; *shares says
// whether that kernel finished only with the copy.  Two passes, the first warms up.
lmc_status_t shares_a_queue(lmc_ctx *c, hipStream_t busy, bool by_kernel, hipStream_t other, uint8_t *devbuf,
                            uint64_t nbytes, hipEvent_t a0, hipEvent_t a1, hipEvent_t k1, bool *shares) {
    float t_copy = 0.f, t_kernel = 0.f;
    for (int pass = 0; pass < 2; pass++) {
        const hipError_t steps[] = {
            hipEventRecord(a0, busy),
            by_kernel ? lmc::launch_copy_rect(devbuf, nbytes, c->pool_dev, nbytes, nbytes, 1,
                                              c->link_groups ? c->link_groups : 64u, busy)
                      : hipMemcpyAsync(devbuf, c->pool, nbytes, hipMemcpyHostToDevice, busy),
            hipEventRecord(a1, busy),
            lmc::launch_fill(devbuf + nbytes, 0, 256, other),
            hipEventRecord(k1, other),
            hipEventSynchronize(a1),
            hipEventSynchronize(k1),
            hipEventElapsedTime(&t_copy, a0, a1),
            hipEventElapsedTime(&t_kernel, a0, k1),
        };
        for (hipError_t x : steps)
            if (x != hipSuccess) {
                c->last_hip_error = int32_t(x);
                (void)hipGetLastError();
                return LMC_ERR_HIP;
            }
    }
    *shares = t_kernel > 0.5f * t_copy;
    return LMC_OK;
}

// Puts the library's six streams on hardware queues of its choosing.  HIP gives every
// stream one of a few hardware queues when the stream is created (four by default, the
// least used one first) and a queue runs its entries in order: a stream stands still not
// only while a copy of a queue-mate runs but also while a queue-mate *waits* for an event,
// so a scatter launch waiting for its group's copy holds up a gather behind it.  Left as
// created, which streams share is a matter of how many streams the process made before;
// measured on the 10 GiB request with a store and a retrieve running together: 63, 72 or
// 100 GB/s summed, by arrangement alone.  The plan: the two kernel streams and the first
// copy stream of each direction on four different queues, so that the four streams of a
// full-duplex transfer never wait for each other.  A second copy stream must not sit
// behind the first one of its direction (the steps of a layer-wise transfer alternate
// between the two so that one step's copy starts while the other's is being retired: in
// one queue that gains nothing, 52.7 instead of 56.2 GB/s for a retrieve at four layers a
// step), nor behind the kernel stream of its own direction (whose waits would hold it up),
// nor with a copy stream of the other direction (the copies of a two-way transfer would
// take turns).  So each joins the kernel stream of the *other* direction, which a one-way
// transfer leaves idle: the second host-to-device stream the gather stream's queue, the
// second device-to-host stream the scatter stream's.  other_direction_busy() keeps the
// second streams out of a transfer that finds the other direction at work.  With
// fewer queues a kernel stream joins the first copy stream of the other direction; with six
// or more every stream has its own.  Streams are told apart by shares_a_queue(); candidates
// are created until the plan can be met (at most 16, the unused ones are destroyed); if it
// cannot be, or anything fails, the streams stay as created.  Streams of the caller are the
// caller's to place: lmc_probe_stream.  Needs an idle context.
void arrange_streams(lmc_ctx *c) {
    // scratch: a staging buffer of the store ring, which nothing is using (no allocation here)
    if (c->store_ring.buf.empty() || c->store_ring.buf_bytes < 512) return;
    const uint64_t pool_bytes = uint64_t(c->n_pool_slots) * uint64_t(c->chunk_bytes);
    const uint64_t nbytes =
        std::min({uint64_t(32) << 20, pool_bytes, c->store_ring.buf_bytes - 256}) / 256 * 256;
    if (nbytes < (uint64_t(8) << 20)) return;   // too short a copy to tell waiting from running
    uint8_t *devbuf = c->store_ring.buf[0];
    hipEvent_t a0 = nullptr, a1 = nullptr, k1 = nullptr;
    // roles in the order in which they get a queue of their own while queues last
    hipStream_t *const role[6] = {&c->s_h2d, &c->s_d2h, &c->s_scatter, &c->s_gather, &c->s_h2d2, &c->s_d2h2};
    const int partner[6] = {0, 1, 1, 0, 3, 2};   // whose queue to join when none is left
    std::vector<hipStream_t> cand;
    for (hipStream_t *r : role) cand.push_back(*r);
    std::vector<int> queue_of;        // per candidate: number of its hardware queue, as found
    std::vector<size_t> first_in;     // per queue found: its first candidate
    int pick[6] = {0, 1, 2, 3, 4, 5};
    bool ok = get_event(c, true, &a0) == LMC_OK && get_event(c, true, &a1) == LMC_OK && get_event(c, true, &k1) == LMC_OK;
    bool met = false;
    while (ok && !met) {
        // place the candidates not yet placed
        while (ok && queue_of.size() < cand.size()) {
            const size_t i = queue_of.size();
            int q = -1;
            for (size_t k = 0; ok && q < 0 && k < first_in.size(); k++) {
                bool shares = false;
                ok = shares_a_queue(c, cand[first_in[k]], false, cand[i], devbuf, nbytes, a0, a1, k1, &shares) == LMC_OK;
                if (shares) q = int(k);
            }
            if (q < 0) {
                q = int(first_in.size());
                first_in.push_back(i);
            }
            queue_of.push_back(q);
        }
        if (!ok) break;
        // try the plan with what there is
        std::vector<char> taken(cand.size(), 0);
        int role_queue[6], next_queue = 0;
        met = true;
        for (int r = 0; r < 6 && met; r++) {
            const int want = next_queue < int(first_in.size()) ? next_queue++ : role_queue[partner[r]];
            role_queue[r] = want;
            met = false;
            for (size_t i = 0; i < cand.size() && !met; i++)
                if (!taken[i] && queue_of[i] == want) {
                    taken[i] = 1;
                    pick[r] = int(i);
                    met = true;
                }
        }
        // A queue that other streams of the process use much is handed out last: with fewer
        // than six queues seen, look at a dozen streams before believing the count.
        if (met && first_in.size() < 6 && cand.size() < 12) met = false;
        if (!met) {
            hipStream_t fresh = nullptr;
            if (cand.size() >= 16 || hipStreamCreateWithFlags(&fresh, hipStreamNonBlocking) != hipSuccess) break;
            cand.push_back(fresh);
        }
    }
    (void)hipDeviceSynchronize();
    std::vector<char> keep(cand.size(), 0);
    if (ok && met) {
        hipStream_t chosen[6];
        for (int r = 0; r < 6; r++) chosen[r] = cand[size_t(pick[r])];
        for (int r = 0; r < 6; r++) {
            *role[r] = chosen[r];
            keep[size_t(pick[r])] = 1;
        }
    } else {
        for (size_t i = 0; i < 6; i++) keep[i] = 1;
    }
    // The streams not chosen live on, unused, until the context goes: events that were
    // recorded on them are in circulation (the three of the test above, and after a
    // repeated arrangement every event of the rings), and the runtime looks up the stream an
    // event was last recorded on when the event is queried or waited for.  With the stream
    // destroyed, hipEventQuery now and then answered "operation not permitted when stream is
    // capturing" from whatever lay in the freed stream's place.
    for (size_t i = 0; i < cand.size(); i++)
        if (!keep[i]) c->retired_streams.push_back(cand[i]);
    for (hipEvent_t ev : {a0, a1, k1})
        if (ev) c->free_time_events.push_back(ev);
    (void)hipGetLastError();
}

void destroy_ctx(lmc_ctx *c) {
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

}  // namespace

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

// A slot for a new chunk: the lowest free one; with LMC_FLAG_EVICT_LRU and a full pool
// the least recently used chunk that may go gives up its slot.  -1: no room.
static int64_t take_slot(lmc_ctx *c, uint64_t id) {
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
                                 bool edge_group, bool direct, bool on_second_stream = false) {
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
        hipStream_t second = (two_copy_streams && several_runs(&new_slot[j0], int64_t(k))) ? other : nullptr;
        if (second) HIPCHK(c, hipStreamWaitEvent(second, ring.filled[b], 0));
        bool used_second = false;
        rc = copy_group(c, true, buf, view.chunk_stride, &new_slot[j0], int64_t(k), pool_off,
                        view.chunk_stride, copies, second, &used_second);
        if (rc != LMC_OK) return rc;
        // the group's copy stream stands for the whole group: it ends after the other stream's copies
        if (used_second && (rc = order_after(c, copies, second)) != LMC_OK) return rc;
        if (c->cfg.flags & LMC_FLAG_POISON_STAGING)
            HIPCHK(c, lmc::launch_fill(buf, 0xA5, uint64_t(k) * view.chunk_stride, copies));
        HIPCHK(c, hipEventRecord(ring.drained[b], copies));
        ring.used[b] = 1;
        if ((rc = force_sync(c, copies)) != LMC_OK) return rc;
        j0 += k;
    }
    return LMC_OK;
}

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
    std::vector<int64_t> new_chunk;
    const bool fits = admit_new_chunks(c, ids, n_chunks, &op, &new_chunk);
    c->stats.chunks_stored += new_chunk.size();
    const bool direct = (c->cfg.flags & LMC_FLAG_DIRECT) != 0 ||
                        int64_t(new_chunk.size()) * c->chunk_bytes <= c->direct_store_below;
    rc = direct ? LMC_OK : ring_reslot(c, c->store_ring, c->store_ring.buf_bytes, c->s_gather, c->s_d2h, nullptr, c->s_d2h2);
    if (rc == LMC_OK)
        rc = store_groups(c, lmc::bulk_view(c->kg), 0, ptrs, slot_mapping, new_chunk, op.slots,
                          c->cfg.staging_chunks, true, direct);
    if (rc == LMC_OK)
        rc = finish_op(c, std::move(op), direct ? c->s_gather : c->s_d2h, !new_chunk.empty(), ticket_out);
    if (rc != LMC_OK) {
        abort_store(c, op.slots);   // finish_op registers as its last step: op is still whole
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
                          op->slots, cap, false, direct, on_second);
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

static lmc_status_t device_only(lmc_ctx_t *c, bool gather, void *const *kv_layers,
                                const int64_t *slot_mapping, int64_t n_chunks, uint8_t *staging,
                                void *stream) {
    if (!c || n_chunks < 0 || !kv_layers || (n_chunks > 0 && (!slot_mapping || !staging)))
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    if (reinterpret_cast<uintptr_t>(staging) % c->kg.vec) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
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

lmc_status_t lmc_gather(lmc_ctx_t *c, void *const *kv_layers, const int64_t *slot_mapping,
                        int64_t n_chunks, void *staging_dev, void *stream) {
    return device_only(c, true, kv_layers, slot_mapping, n_chunks, static_cast<uint8_t *>(staging_dev), stream);
}

lmc_status_t lmc_scatter(lmc_ctx_t *c, const void *staging_dev, const int64_t *slot_mapping,
                         int64_t n_chunks, void *const *kv_layers, void *stream) {
    return device_only(c, false, kv_layers, slot_mapping, n_chunks,
                       static_cast<uint8_t *>(const_cast<void *>(staging_dev)), stream);
}

lmc_status_t lmc_store_static(lmc_ctx_t *c, void *const *kv_layers, const int64_t *slot_mapping,
                              int64_t n_chunks, void *host_dst, void *stream) {
    if (!c || n_chunks < 0 || !kv_layers || (n_chunks > 0 && (!slot_mapping || !host_dst)))
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    if (c->cfg.device >= kMaxDevices) return LMC_ERR_INVAL;
    uint8_t *const stage = static_scratch_of(c->cfg.device);   // looked up by lmc_create
    if (stage == nullptr) return LMC_ERR_HIP;
    const lmc_kv_geom_t &geom = c->cfg.geom;
    const uint64_t cb = uint64_t(c->chunk_bytes);
    const uint64_t layer_bytes = uint64_t(geom.num_planes) * c->kg.plane_bytes;
    // the unit that must fit into the scratch array is one layer of one chunk
    if (layer_bytes > LMC_STATIC_SCRATCH_BYTES) return LMC_ERR_INVAL;
    if (n_chunks == 0) return LMC_OK;
    // the destination must be pinned host memory: the runtime stages a copy to pageable
    // memory through buffers of its own, which it may have to allocate
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host_dst) != hipSuccess || attr.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return LMC_ERR_INVAL;
    }
    lmc::LayerPtrs ptrs;
    lmc_status_t rc = build_layer_ptrs(c, kv_layers, &ptrs);
    if (rc != LMC_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t CT = geom.chunk_tokens;
    if ((rc = validate_slots(c, slot_mapping, n_chunks * CT, s)) != LMC_OK) return rc;
    uint8_t *dst = static_cast<uint8_t *>(host_dst);
    // One piece at a time through the scratch array, kernel then copy, all on the caller's
    // stream: the stream's own order keeps the next kernel off the array until the copy
    // has read it, so no event is needed.  Every byte of a piece is written by its gather
    // (tokens without a page as zeros), so what an earlier call left behind never shows.
    auto piece = [&](const lmc::LaunchView &view, const int64_t *slots, uint32_t k, uint8_t *to,
                     uint64_t bytes) -> lmc_status_t {
        HIPCHK(c, lmc::launch_gather(c->kg, view, c->shape, ptrs, slots, k, stage, c->bad_flag_dev, s));
        HIPCHK(c, hipMemcpyAsync(to, stage, size_t(bytes), hipMemcpyDeviceToHost, s));
        c->stats.gather_launches++;
        c->stats.bytes_gathered += bytes;
        c->stats.bytes_d2h += bytes;
        return LMC_OK;
    };
    if (cb <= LMC_STATIC_SCRATCH_BYTES) {
        // whole chunks, as many per launch as the array holds
        const lmc::LaunchView view = lmc::bulk_view(c->kg);
        const int64_t per = std::min<int64_t>(int64_t(LMC_STATIC_SCRATCH_BYTES / cb),
                                              int64_t(lmc::max_chunks_per_launch(c->kg, view)));
        for (int64_t i0 = 0; i0 < n_chunks; i0 += per) {
            const int64_t k = std::min(per, n_chunks - i0);
            if ((rc = piece(view, slot_mapping + i0 * CT, uint32_t(k), dst + uint64_t(i0) * cb, uint64_t(k) * cb)) != LMC_OK)
                return rc;
        }
    } else {
        // a chunk larger than the array goes a few layers at a time: the layers of a chunk
        // are consecutive in it, so each piece is still one contiguous copy
        const int32_t per = int32_t(std::min<uint64_t>(LMC_STATIC_SCRATCH_BYTES / layer_bytes, uint64_t(geom.num_layers)));
        for (int64_t i = 0; i < n_chunks; i++)
            for (int32_t l0 = 0; l0 < geom.num_layers; l0 += per) {
                const int32_t nl = std::min(per, geom.num_layers - l0);
                const lmc::LaunchView view = lmc::layer_view(c->kg, uint32_t(geom.num_planes), uint32_t(l0), uint32_t(nl));
                if ((rc = piece(view, slot_mapping + i * CT, 1, dst + uint64_t(i) * cb + uint64_t(l0) * layer_bytes,
                                uint64_t(nl) * layer_bytes)) != LMC_OK)
                    return rc;
            }
    }
    return LMC_OK;
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

static lmc_status_t measure_link(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, bool by_kernel,
                                 double *h2d_out, double *d2h_out) {
    if (!c || !h2d_out || !d2h_out || reps < 1 || nbytes == 0) return LMC_ERR_INVAL;
    if (by_kernel && (nbytes % 16) != 0) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    if (nbytes > uint64_t(c->n_pool_slots) * uint64_t(c->chunk_bytes)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    HIPCHK(c, hipDeviceSynchronize());
    reap(c);
    uint8_t *devbuf = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&devbuf), nbytes);
    if (e != hipSuccess) {
        c->last_hip_error = int32_t(e);
        (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
        return LMC_ERR_NOMEM;
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    lmc_status_t rc = get_event(c, true, &e0);
    if (rc == LMC_OK) rc = get_event(c, true, &e1);
    double best[2] = {0.0, 0.0};
    // upload first, then download the same bytes: the pool ends as it started
    for (int dir = 0; dir < 2 && rc == LMC_OK; dir++) {
        hipStream_t s = dir == 0 ? c->s_h2d : c->s_d2h;
        for (int r = 0; r < reps + 1; r++) {  // first pass warms up
            hipError_t a = hipEventRecord(e0, s);
            const uint32_t groups = c->link_groups ? c->link_groups : 64u;
            hipError_t b = by_kernel
                ? (dir == 0 ? lmc::launch_copy_rect(devbuf, nbytes, c->pool_dev, nbytes, nbytes, 1, groups, s)
                            : lmc::launch_copy_rect(c->pool_dev, nbytes, devbuf, nbytes, nbytes, 1, groups, s))
                : (dir == 0 ? hipMemcpyAsync(devbuf, c->pool, nbytes, hipMemcpyHostToDevice, s)
                            : hipMemcpyAsync(c->pool, devbuf, nbytes, hipMemcpyDeviceToHost, s));
            hipError_t d = hipEventRecord(e1, s);
            hipError_t f = hipEventSynchronize(e1);
            float ms = 0.f;
            hipError_t g = hipEventElapsedTime(&ms, e0, e1);
            for (hipError_t x : {a, b, d, f, g})
                if (x != hipSuccess) {
                    c->last_hip_error = int32_t(x);
                    (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
                    rc = LMC_ERR_HIP;
                }
            if (rc != LMC_OK) break;
            if (r > 0 && ms > 0.f) best[dir] = std::max(best[dir], double(nbytes) / (double(ms) * 1e6));
        }
    }
    if (e0) c->free_time_events.push_back(e0);
    if (e1) c->free_time_events.push_back(e1);
    (void)hipFree(devbuf);
    *h2d_out = best[0];
    *d2h_out = best[1];
    return rc;
}

lmc_status_t lmc_measure_link(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, double *h2d_out,
                              double *d2h_out) {
    return measure_link(c, nbytes, reps, false, h2d_out, d2h_out);
}

lmc_status_t lmc_measure_link_kernel(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, double *h2d_out,
                                     double *d2h_out) {
    return measure_link(c, nbytes, reps, true, h2d_out, d2h_out);
}

lmc_status_t lmc_probe_stream(lmc_ctx_t *c, void *stream, uint32_t *mask_out) {
    if (!c || !mask_out) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    HIPCHK(c, hipDeviceSynchronize());
    reap(c);
    const uint64_t pool_bytes = uint64_t(c->n_pool_slots) * uint64_t(c->chunk_bytes);
    const uint64_t nbytes = std::min<uint64_t>(uint64_t(64) << 20, pool_bytes) / 16 * 16;
    uint8_t *devbuf = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&devbuf), nbytes + 256);
    if (e != hipSuccess) {
        c->last_hip_error = int32_t(e);
        (void)hipGetLastError();
        return LMC_ERR_NOMEM;
    }
    hipEvent_t a0 = nullptr, a1 = nullptr, k1 = nullptr;
    lmc_status_t rc = get_event(c, true, &a0);
    if (rc == LMC_OK) rc = get_event(c, true, &a1);
    if (rc == LMC_OK) rc = get_event(c, true, &k1);
    hipStream_t user = static_cast<hipStream_t>(stream);
    const hipStream_t copy_streams[6] = {c->s_h2d, c->s_h2d2, c->s_d2h, c->s_d2h2, c->s_gather, c->s_scatter};
    uint32_t mask = 0;
    for (int i = 0; i < 6 && rc == LMC_OK; i++) {
        // on the two kernel streams: the link-paced kernel that direct mode runs there
        bool shares = false;
        rc = shares_a_queue(c, copy_streams[i], i >= 4, user, devbuf, nbytes, a0, a1, k1, &shares);
        if (rc == LMC_OK && shares) mask |= 1u << i;
    }
    (void)hipDeviceSynchronize();
    for (hipEvent_t ev : {a0, a1})
        if (ev) c->free_time_events.push_back(ev);
    // k1 was recorded on the caller's stream, which the caller may destroy while the event
    // is still in circulation here (see arrange_streams): it is not kept
    if (k1) {
        c->all_events.erase(std::remove(c->all_events.begin(), c->all_events.end(), k1), c->all_events.end());
        (void)hipEventDestroy(k1);
    }
    (void)hipFree(devbuf);
    (void)hipGetLastError();
    *mask_out = mask;
    return rc;
}

static lmc_status_t measure_duplex(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, uint32_t by_kernel,
                                   double *gbps_out) {
    // bits 0-1: which direction the copy kernel makes; bits 8-15: in how many consecutive
    // pieces each direction moves its bytes (0 = 1), as the pipelines do group by group
    const uint32_t pieces = std::max<uint32_t>(1u, (by_kernel >> 8) & 0xFFu);
    by_kernel &= ~0xFF00u;
    if (!c || !gbps_out || reps < 1 || nbytes == 0 || by_kernel > 3) return LMC_ERR_INVAL;
    if (nbytes % (uint64_t(pieces) * 16) != 0) return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    if (2 * nbytes > uint64_t(c->n_pool_slots) * uint64_t(c->chunk_bytes)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    DeviceScope dev(c);
    HIPCHK(c, hipDeviceSynchronize());
    reap(c);
    uint8_t *up = nullptr, *down = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&up), nbytes) != hipSuccess) return LMC_ERR_NOMEM;
    if (hipMalloc(reinterpret_cast<void **>(&down), nbytes) != hipSuccess) {
        (void)hipFree(up);
        return LMC_ERR_NOMEM;
    }
    hipEvent_t e0 = nullptr, e1 = nullptr, e2 = nullptr;
    lmc_status_t rc = get_event(c, true, &e0);
    if (rc == LMC_OK) rc = get_event(c, true, &e1);
    if (rc == LMC_OK) rc = get_event(c, true, &e2);
    double best = 0.0;
    auto ok = [&](hipError_t e) {
        if (e != hipSuccess && rc == LMC_OK) {
            c->last_hip_error = int32_t(e);
            (void)hipGetLastError();  // the runtime keeps a failure as its "last error": take it back
            rc = LMC_ERR_HIP;
        }
    };
    // the second half of the region is uploaded first and downloaded unchanged in every
    // pass, so the pool ends as it started
    if (rc == LMC_OK) ok(hipMemcpy(down, c->pool + nbytes, nbytes, hipMemcpyHostToDevice));
    for (int r = 0; r < reps + 1 && rc == LMC_OK; r++) {
        ok(hipEventRecord(e0, c->s_h2d));
        ok(hipStreamWaitEvent(c->s_d2h, e0, 0));           // both directions start together
        const uint32_t groups = c->link_groups ? c->link_groups : 64u;
        const uint64_t piece = nbytes / pieces;
        for (uint64_t o = 0; o < nbytes; o += piece) {
            ok((by_kernel & 1u) ? lmc::launch_copy_rect(up + o, piece, c->pool_dev + o, piece, piece, 1, groups, c->s_h2d)
                                : hipMemcpyAsync(up + o, c->pool + o, piece, hipMemcpyHostToDevice, c->s_h2d));
            ok((by_kernel & 2u) ? lmc::launch_copy_rect(c->pool_dev + nbytes + o, piece, down + o, piece, piece, 1, groups, c->s_d2h)
                                : hipMemcpyAsync(c->pool + nbytes + o, down + o, piece, hipMemcpyDeviceToHost, c->s_d2h));
        }
        ok(hipEventRecord(e1, c->s_d2h));
        ok(hipStreamWaitEvent(c->s_h2d, e1, 0));
        ok(hipEventRecord(e2, c->s_h2d));                  // after both
        ok(hipEventSynchronize(e2));
        float ms = 0.f;
        ok(hipEventElapsedTime(&ms, e0, e2));
        if (rc == LMC_OK && r > 0 && ms > 0.f) best = std::max(best, 2.0 * double(nbytes) / (double(ms) * 1e6));
    }
    for (hipEvent_t e : {e0, e1, e2})
        if (e) c->free_time_events.push_back(e);
    (void)hipFree(up);
    (void)hipFree(down);
    *gbps_out = best;
    return rc;
}

lmc_status_t lmc_measure_link_duplex(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, double *gbps_out) {
    return measure_duplex(c, nbytes, reps, 0, gbps_out);
}

lmc_status_t lmc_measure_link_duplex_kernel(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, uint32_t by_kernel,
                                            double *gbps_out) {
    return measure_duplex(c, nbytes, reps, by_kernel, gbps_out);
}

lmc_status_t lmc_copy(lmc_ctx_t *c, void *dst, const void *src, uint64_t nbytes, void *stream) {
    if (!c || !dst || !src || (nbytes % 16) != 0 || (reinterpret_cast<uintptr_t>(dst) % 16) != 0 ||
        (reinterpret_cast<uintptr_t>(src) % 16) != 0)
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    DeviceScope dev(c);
    HIPCHK(c, lmc::launch_copy(static_cast<uint8_t *>(dst), static_cast<const uint8_t *>(src), nbytes,
                               static_cast<hipStream_t>(stream)));
    return LMC_OK;
}

lmc_status_t lmc_copy_tiles(lmc_ctx_t *c, void *dst, const uint32_t *dst_order, const void *src,
                            const uint32_t *src_order, uint64_t n_tiles, uint32_t mode, void *stream) {
    if (!c || !dst || !src || mode > 2 || n_tiles > 0x7FFFFFFFull ||
        (reinterpret_cast<uintptr_t>(dst) % 16) != 0 || (reinterpret_cast<uintptr_t>(src) % 16) != 0)
        return LMC_ERR_INVAL;
    if (!c->has_device) return LMC_ERR_NODEVICE;
    DeviceScope dev(c);
    // mode 1 needs somewhere to pretend to write to: the flag block's last words, seen by the GPU
    uint8_t *sink = reinterpret_cast<uint8_t *>(c->bad_flag_dev + 12);
    HIPCHK(c, lmc::launch_copy_tiles(static_cast<uint8_t *>(dst), dst_order, static_cast<const uint8_t *>(src),
                                     src_order, uint32_t(n_tiles), mode, sink, static_cast<hipStream_t>(stream)));
    return LMC_OK;
}

lmc_status_t lmc_tune(lmc_ctx_t *c, const char *key, int64_t value) {
    if (!c || !key || value < 0) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    const std::string k(key);
    if (k == "timing" && value <= 1) {
        c->cfg.flags = value ? (c->cfg.flags | LMC_FLAG_TIMING) : (c->cfg.flags & ~LMC_FLAG_TIMING);
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
