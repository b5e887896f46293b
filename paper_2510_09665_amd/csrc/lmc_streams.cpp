// liblmc: which hardware queues streams sit in (the library's own: arranged; the caller's: probed).
#include "lmc_ctx.hpp"

namespace lmci {

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
    // the test tells waiting from running by the clock: nothing else should be running
    (void)hipDeviceSynchronize();
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

}  // namespace lmci

using namespace lmci;

extern "C" {

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

}  // extern "C"
