// liblmc: the one entry point that allocates nothing, and the static device array behind it.
#include "lmc_ctx.hpp"

// Device memory for the one entry point that must not allocate (lmc_store_static): the
// staging buffer of that call.  Every GPU the library's code is loaded on holds its own
// copy of this array, at its own address, until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; the address that kernels and copies
// use is the one looked up per device in static_scratch_at.
static __device__ __align__(256) uint8_t scratch[LMC_STATIC_SCRATCH_BYTES];

namespace lmci {

constexpr int kMaxDevices = 64;
static uint8_t *static_scratch_at[kMaxDevices];   // per device ordinal; null = not looked up yet
static std::mutex static_scratch_mu;

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

}  // namespace lmci

using namespace lmci;

extern "C" {

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

}  // extern "C"
