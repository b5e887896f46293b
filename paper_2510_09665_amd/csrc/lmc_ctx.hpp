// Internal to liblmc: the context behind lmc_ctx_t and what its translation units share
// (lmc_ctx.cpp: life cycle, index calls, waiting; lmc_pipeline.cpp: store / retrieve;
// lmc_streams.cpp: hardware queues; lmc_measure.cpp: measurement aids; lmc_static.cpp: the
// entry point that allocates nothing).  Not part of the C ABI (include/lmc.h).
#ifndef LMC_CTX_HPP
#define LMC_CTX_HPP
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

namespace lmci {

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

// One timed step of a pipeline: a kernel launch (LMC_FLAG_TIMING, LMC_FLAG_TRACE) or the
// copies of one group (LMC_FLAG_TRACE), between two timing events.
struct Timing {
    hipEvent_t start, stop;
    int32_t stage;        // LMC_STAGE_*
    uint64_t ticket;      // the operation the step belongs to, 0 = none
    int32_t chunks;
    uint64_t bytes;
};

struct CopyTiming {   // a large device-to-host copy by the runtime, watched by the guard
    hipEvent_t start, stop;
    uint64_t bytes;
};

}  // namespace lmci

using lmci::CopyTiming;
using lmci::Op;
using lmci::Ring;
using lmci::Timing;

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
    // the runtime's are slow (lmc_guard.hpp).  On unless switched off (lmc_tune "d2h_guard"):
    // in a mix of stores and retrieves of many requests the runtime's copies to the host
    // collapse now and then (whole stores at 12.7 GB/s), and the mix runs in 3.2 s with the
    // guard against 4.4-5.2 s without; on the one-way 10 GiB request it costs nothing when
    // the runtime is healthy (one pair of event markers per group) and lifts a fresh
    // process's slow first seconds from 44.5 to 54.5 GB/s.
    bool d2h_guard_on = true;
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
    // LMC_FLAG_TRACE: finished steps, oldest first, at most kTraceCap; device time counts from trace_epoch
    std::deque<lmc_trace_rec_t> trace;
    uint64_t trace_dropped = 0;
    hipEvent_t trace_epoch = nullptr;
    uint64_t cur_ticket = 0;   // the operation whose steps are being enqueued (for the trace)
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

namespace lmci {

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
constexpr size_t kTraceCap = size_t(1) << 16;

// lmc_ctx.cpp
lmc_status_t get_event(lmc_ctx *c, bool timing, hipEvent_t *out);
lmc_status_t build_layer_ptrs(const lmc_ctx *c, void *const *kv_layers, lmc::LayerPtrs *out);
Op *find_op(lmc_ctx *c, uint64_t ticket);
double seconds_now(const lmc_ctx *c);
void recycle(lmc_ctx *c, hipEvent_t e);
void reap(lmc_ctx *c);
lmc_status_t order_after(lmc_ctx *c, hipStream_t waiter, hipStream_t stream);
lmc_status_t order_after_caller(lmc_ctx *c, hipStream_t waiter, hipStream_t user);
bool other_direction_busy(lmc_ctx *c, bool for_store);
lmc_status_t validate_slots(lmc_ctx *c, const int64_t *slot_mapping, int64_t n_tokens,
                            hipStream_t stream);
lmc_status_t force_sync(lmc_ctx *c, hipStream_t s);
lmc_status_t trace_begin(lmc_ctx *c, hipStream_t stream, hipEvent_t *start);
lmc_status_t trace_end(lmc_ctx *c, hipStream_t stream, hipEvent_t start, int32_t stage, int64_t chunks, uint64_t bytes);
void begin_use(lmc_ctx *c, const uint64_t *ids, int64_t n);
void end_use(lmc_ctx *c, const uint64_t *ids, int64_t n);
int64_t take_slot(lmc_ctx *c, uint64_t id);
lmc_status_t free_ring(Ring &r);
lmc_status_t make_ring(lmc_ctx *c, Ring &r);
// lmc_pipeline.cpp
lmc_status_t timed_launch(lmc_ctx *c, bool gather, const lmc::LaunchView &view,
                          const lmc::LayerPtrs &ptrs, const int64_t *slots, uint32_t n_chunks,
                          uint8_t *staging, hipStream_t stream);
// lmc_streams.cpp
lmc_status_t shares_a_queue(lmc_ctx *c, hipStream_t busy, bool by_kernel, hipStream_t other, uint8_t *devbuf,
                            uint64_t nbytes, hipEvent_t a0, hipEvent_t a1, hipEvent_t k1, bool *shares);
void arrange_streams(lmc_ctx *c);
// lmc_static.cpp
hipError_t resolve_static_scratch(int device);
uint8_t *static_scratch_of(int device);

}  // namespace lmci

#endif  // LMC_CTX_HPP
