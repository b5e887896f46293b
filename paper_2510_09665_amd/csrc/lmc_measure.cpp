// liblmc: measurement aids of the C ABI (link peaks one-way and two-way, plain copies as yardsticks).
#include "lmc_ctx.hpp"

namespace lmci {

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

}  // namespace lmci

using namespace lmci;

extern "C" {

lmc_status_t lmc_measure_link(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, double *h2d_out,
                              double *d2h_out) {
    return measure_link(c, nbytes, reps, false, h2d_out, d2h_out);
}

lmc_status_t lmc_measure_link_kernel(lmc_ctx_t *c, uint64_t nbytes, int32_t reps, double *h2d_out,
                                     double *d2h_out) {
    return measure_link(c, nbytes, reps, true, h2d_out, d2h_out);
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

}  // extern "C"
