// Internal launch interface of the device kernels (gfx950).  Host code fills a
// KernelGeom once per context; the launchers check nothing: callers have validated
// shapes, alignment and pointers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace lmc {

constexpr int kMaxLayers = 160;
constexpr int kMaxLayerPlanes = 2 * kMaxLayers;

// Base pointer of every (layer, plane), index l*n_planes + p.  The table travels by
// value as a kernel argument: no device-side table to allocate, upload or keep alive,
// and the kernels read it with scalar loads.
struct LayerPtrs {
    uint8_t *p[kMaxLayerPlanes];
};

// What the gather / scatter kernels need to know, precomputed on the host.
// A "row" is one token of one layer and plane in the chunk: vec_per_row vectors of
// `vec` bytes.  In the pages a row is runs_per_row runs of vec_per_run vectors; when a
// token's heads are contiguous the host folds them into a single run.
struct KernelGeom {
    int64_t block_stride, token_stride, run_stride;  // bytes
    uint64_t row_stride_lp;   // chunk_tokens * row bytes: distance between layer-planes in a chunk
    uint64_t chunk_bytes;
    uint32_t n_slots;         // num_blocks * block_size
    uint32_t block_size;
    int32_t block_shift;      // log2(block_size), or -1 when it is not a power of two
    uint32_t chunk_tokens;
    uint32_t vec_per_run, runs_per_row, vec_per_row;
    uint32_t pairs_per_chunk; // chunk_tokens * vec_per_row
    uint32_t n_layer_planes;  // num_layers * num_planes
    uint32_t vec;             // bytes per lane access: 16, 8, 4, 2 or 1
};

struct LaunchShape {
    uint32_t lp_per_block;    // layer-planes walked by one workgroup
    bool nt_load, nt_store;
};

// pages -> chunks [first_chunk, first_chunk + n_chunks) of the slot mapping, written
// back to back from `staging`.  bad_flag: device-visible int set to 1 on a slot >= n_slots.
hipError_t launch_gather(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                         const int64_t *slot_mapping, uint32_t n_chunks, uint8_t *staging,
                         int32_t *bad_flag, hipStream_t stream);
hipError_t launch_scatter(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                          const int64_t *slot_mapping, uint32_t n_chunks, const uint8_t *staging,
                          int32_t *bad_flag, hipStream_t stream);
// *bad_flag = 1 if any of the n slots is >= n_slots
hipError_t launch_check_slots(const int64_t *slot_mapping, uint64_t n, uint32_t n_slots,
                              int32_t *bad_flag, hipStream_t stream);
hipError_t launch_copy(uint8_t *dst, const uint8_t *src, uint64_t nbytes, hipStream_t stream);
hipError_t launch_fill(uint8_t *dst, uint8_t value, uint64_t nbytes, hipStream_t stream);

// largest number of chunks one launch may cover (32-bit pair index)
uint32_t max_chunks_per_launch(const KernelGeom &g);

}  // namespace lmc
