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

// Division of a 31-bit value by a run-time constant as multiply-high and shift.
// With l = ceil(log2 d), mul = floor(2^(31+l) / d) + 1 and shift = l - 1, the quotient
// mulhi(n, mul) >> shift is exact for every n < 2^31 (the error term n / 2^(31+l) stays
// below 1/d).  d == 1 is flagged by mul == 0.
struct FastDiv {
    uint32_t mul, shift, d;
#if defined(__HIPCC__)
    __host__ __device__
#endif
    uint32_t div(uint32_t n) const {
        return mul == 0 ? n : uint32_t((uint64_t(n) * mul) >> 32) >> shift;
    }
};
FastDiv make_fastdiv(uint32_t d);  // d >= 1

// What the gather / scatter kernels need to know, precomputed on the host.
// A "plane" is one (layer, plane) of one chunk: chunk_tokens rows of vec_per_row vectors
// of `vec` bytes, contiguous in the chunk.  In the pages a row is runs_per_row runs of
// vec_per_run vectors; when a token's heads are contiguous the host folds them into a
// single run.  A workgroup copies one tile of 256 consecutive vectors of a plane.
struct KernelGeom {
    int64_t block_stride, token_stride, run_stride;  // bytes
    uint64_t plane_bytes;     // chunk_tokens * row bytes
    uint64_t chunk_bytes;
    uint32_t n_slots;         // num_blocks * block_size
    uint32_t chunk_tokens;
    uint32_t vec_per_plane;   // chunk_tokens * vec_per_row
    uint32_t runs_per_row;
    uint32_t n_layer_planes;  // num_layers * num_planes
    uint32_t vec;             // bytes per lane access: 16, 8, 4, 2 or 1
    FastDiv by_tiles_per_plane, by_vec_per_row, by_vec_per_run, by_block_size;
};

// Which part of every chunk one launch moves, and how the chunks lie in the staging
// buffer.  Bulk mode moves all layer-planes and chunks are chunk_bytes apart; layer-wise
// mode moves the planes of a few consecutive layers and packs just those.
struct LaunchView {
    FastDiv by_n_lp;        // layer-planes per chunk in this launch
    uint32_t lp_base;       // first layer-plane (index into LayerPtrs)
    uint64_t chunk_stride;  // bytes between consecutive chunks in the staging buffer
};

struct LaunchShape {
    bool nt_load, nt_store;   // non-temporal hints on the streaming loads / stores
    uint32_t xcd_run;         // workgroup ids are permuted so that each of the 8 XCDs
                              // takes runs of this many (rounded down to a power of
                              // two) consecutive tiles; 0 = off
    uint32_t ordered_group_rows;  // scatter in destination order: rows (tokens) per group, see
                                  // launch_scatter_ordered; 0 = one group, the launch goes plane by plane
    uint32_t paced_groups;    // 0: one tile per workgroup (HBM-bound launches); n > 0: a
                              // fixed grid of n workgroups that take tiles in turn, for
                              // launches whose other side is host memory
};

// pages -> n_chunks chunks of the slot mapping, written back to back from `staging`
// (gather), or the reverse (scatter).  bad_flag: device-visible int set to 1 on a slot
// >= n_slots.  start / stop: optional events (timing enabled) that receive the
// kernel's own begin and end time stamps; no marker is put on the stream for them.
hipError_t launch_gather(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                         const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                         uint8_t *staging, int32_t *bad_flag, hipStream_t stream,
                         hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_scatter(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                          const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                          const uint8_t *staging, int32_t *bad_flag, hipStream_t stream,
                          hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
// Scatter in the order of the destination: the rows of the launch are visited in ascending
// slot order, plane by plane (see lmc_kernels.hip).  The order is built on the device in
// scratch memory the caller provides: token_at (order_table_words() words), counts
// (order_count_words() words), pairs (one per token of the launch), n_rows (one word).
// One scratch set serves one launch at a time.
constexpr uint32_t kMaxOrderedSlots = 1u << 24;     // 64 MiB of table at most
struct OrderScratch {
    uint32_t *token_at, *counts, *n_rows;
    uint2 *pairs;
};
uint64_t order_table_words(const KernelGeom &g);
uint64_t order_count_words(const KernelGeom &g);
// whether a launch over n_tokens tokens of view v can go this way (32-bit index limits)
bool ordered_scatter_fits(const KernelGeom &g, const LaunchView &v, const LaunchShape &s, uint64_t n_tokens);
// same result as launch_scatter over n_tokens / chunk_tokens chunks
hipError_t launch_scatter_ordered(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                                  const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_tokens,
                                  const OrderScratch &o, const uint8_t *staging, int32_t *bad_flag,
                                  hipStream_t stream, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
LaunchView bulk_view(const KernelGeom &g);
LaunchView layer_view(const KernelGeom &g, uint32_t planes_per_layer, uint32_t first_layer,
                      uint32_t n_layers);
// *bad_flag = 1 if any of the n slots is >= n_slots
hipError_t launch_check_slots(const int64_t *slot_mapping, uint64_t n, uint32_t n_slots,
                              int32_t *bad_flag, hipStream_t stream);
hipError_t launch_copy(uint8_t *dst, const uint8_t *src, uint64_t nbytes, hipStream_t stream);
// n_tiles tiles of 4 KiB: tile src_order[w] of src to tile dst_order[w] of dst (null = w);
// mode 0 copy, 1 read only, 2 write only; sink: 16 bytes of device memory for mode 1
hipError_t launch_copy_tiles(uint8_t *dst, const uint32_t *dst_order, const uint8_t *src,
                             const uint32_t *src_order, uint32_t n_tiles, uint32_t mode, uint8_t *sink,
                             hipStream_t stream);
// rows x width bytes, rows src_pitch / dst_pitch apart, by `groups` workgroups that take
// tiles in turn (the shape that suits a copy whose one side is pinned host memory).
// Everything must be a multiple of 16 bytes, else hipErrorInvalidValue.
hipError_t launch_copy_rect(uint8_t *dst, uint64_t dst_pitch, const uint8_t *src, uint64_t src_pitch,
                            uint64_t width, uint64_t rows, uint32_t groups, hipStream_t stream);
// Pool slots of the pieces of one copy_pieces launch, by value like LayerPtrs.
constexpr int kMaxPieces = 256;
struct PieceSlots {
    int32_t slot[kMaxPieces];
};
// n_pieces (<= kMaxPieces) pieces of `width` bytes in one launch of the link-paced copy
// kernel: piece i lies at staging + i * stage_pitch and at pool + slot[i] * pool_pitch
// (pool already offset to where a piece starts inside its slot).  to_pool: staging ->
// pool, else pool -> staging.  Everything a multiple of 16 bytes.
hipError_t launch_copy_pieces(uint8_t *pool, uint64_t pool_pitch, uint8_t *staging, uint64_t stage_pitch,
                              uint64_t width, const PieceSlots &slots, uint32_t n_pieces, bool to_pool,
                              uint32_t groups, hipStream_t stream);
hipError_t launch_fill(uint8_t *dst, uint8_t value, uint64_t nbytes, hipStream_t stream);

// largest number of chunks one launch may cover (32-bit workgroup index)
uint32_t max_chunks_per_launch(const KernelGeom &g, const LaunchView &v);

}  // namespace lmc
