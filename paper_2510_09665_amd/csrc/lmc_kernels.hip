// Device kernels of liblmc for gfx950 (MI355X): the paged-KV gather (store direction)
// and scatter (load direction) that the paper's section 5.1 places between the
// engine's pages and the contiguous streaming GPU buffer, plus small helpers.
//
// Both kernels are pure byte movement and HBM-bound; there is no reuse, so neither LDS
// nor MFMA has a role.  What was measured to matter on this part, and shapes the code:
//   - One 16-byte vector per lane and a very large grid.  Occupancy, not unrolling,
//     supplies the bytes in flight: with a handful of VGPRs every SIMD holds its full
//     8 wavefronts.  Unrolled variants that walk several layer-planes per lane were
//     10-15 % slower: their accesses sit power-of-two distances apart (planes of a
//     chunk, layers of the cache) and collide on memory channels.
//   - Workgroup order follows the chunk buffer: tile, then layer-plane, then chunk.
//     The contiguous side of the copy is then swept linearly by the launch as a
//     whole, and the paged side is touched page by page (a page's tokens are
//     consecutive rows).  Ordering by layer-plane first cost 5-10 %.
//   - Non-temporal loads and stores: nothing is read twice.
//   - Index arithmetic (which chunk, plane, token, vector; slot -> block and offset)
//     uses multiply-high division by host-precomputed constants; the workgroup-level
//     part is wave-uniform and runs on the scalar unit.
#include "lmc_kernels.hpp"

#include <hip/hip_ext.h>

#include <algorithm>

namespace lmc {
namespace {

constexpr int kThreads = 256;

template <int N> struct VecOf;
template <> struct VecOf<16> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef unsigned int type; };
template <> struct VecOf<2> { typedef unsigned short type; };
template <> struct VecOf<1> { typedef unsigned char type; };

#define LMC_GLOBAL __attribute__((address_space(1)))

// Addresses are carried as integers (so they can be pinned in scalar registers) and
// dereferenced as global-memory pointers, never as flat ones.
template <typename V, bool NT> __device__ __forceinline__ V load_vec(uint64_t addr) {
    const LMC_GLOBAL V *p = (const LMC_GLOBAL V *)addr;
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <typename V, bool NT> __device__ __forceinline__ void store_vec(uint64_t addr, V v) {
    LMC_GLOBAL V *p = (LMC_GLOBAL V *)addr;
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Keeps a wave-uniform value in scalar registers from this point on.
template <typename T> __device__ __forceinline__ T pin(T v) {
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ FastDiv pin(FastDiv f) {
    f.mul = pin(f.mul);
    f.shift = pin(f.shift);
    f.d = pin(f.d);
    return f;
}

// Everything a tile needs besides its own number, held in scalar registers.
struct TileArgs {
    FastDiv by_tiles, by_lp, by_row, by_run, by_bs;
    uint32_t lp_base, vec_per_plane, chunk_tokens, n_slots, runs_per_row;
    uint64_t chunk_stride, plane_bytes, slots_at, staging_at, bad_flag_at;
    int64_t block_stride, token_stride, run_stride;
};

// Fetches every kernel argument at once, in one batch of scalar loads.  Left alone the
// compiler loads each field just before its first use, which puts four scalar-load
// round trips behind the slot load on every wavefront's critical path.
__device__ __forceinline__ TileArgs fetch_args(const KernelGeom &g, const LaunchView &view,
                                               const int64_t *slot_mapping, uint8_t *staging,
                                               int32_t *bad_flag) {
    TileArgs a;
    a.by_tiles = pin(g.by_tiles_per_plane);
    a.by_lp = pin(view.by_n_lp);
    a.by_row = pin(g.by_vec_per_row);
    a.by_run = pin(g.by_vec_per_run);
    a.by_bs = pin(g.by_block_size);
    a.lp_base = pin(view.lp_base);
    a.chunk_stride = pin(view.chunk_stride);
    a.vec_per_plane = pin(g.vec_per_plane);
    a.chunk_tokens = pin(g.chunk_tokens);
    a.n_slots = pin(g.n_slots);
    a.runs_per_row = pin(g.runs_per_row);
    a.block_stride = pin(g.block_stride);
    a.token_stride = pin(g.token_stride);
    a.run_stride = pin(g.run_stride);
    a.plane_bytes = pin(g.plane_bytes);
    a.slots_at = pin(uint64_t(slot_mapping));
    a.staging_at = pin(uint64_t(staging));
    a.bad_flag_at = pin(uint64_t(bad_flag));
    return a;
}

// One tile (256 consecutive vectors of one plane of one chunk) of the path's copy in
// either direction; lane = one vector r of plane lp of chunk c, token t = r / vec_per_row:
//   GATHER: chunk[c][lp][r] = valid(slot[c][t]) ? page(lp, slot[c][t])[r % vec_per_row] : 0
//   else  : if valid(slot[c][t]):  page(lp, slot[c][t])[r % vec_per_row] = chunk[c][lp][r]
// blk numbers the launch's tiles in chunk-buffer order: tile, then layer-plane, then chunk.
template <int VEC, bool GATHER, bool NT_LD, bool NT_ST>
__device__ __forceinline__ void move_tile(const TileArgs &a, const LayerPtrs &layers, uint32_t blk) {
    typedef typename VecOf<VEC>::type V;
    const uint32_t q = a.by_tiles.div(blk);
    const uint32_t tile = blk - q * a.by_tiles.d;
    const uint32_t c = a.by_lp.div(q);
    const uint32_t lp = q - c * a.by_lp.d;  // plane inside this launch's part of the chunk
    const uint32_t r = tile * kThreads + threadIdx.x;
    if (r >= a.vec_per_plane) return;
    const uint32_t t = a.by_row.div(r);
    const uint32_t w = r - t * a.by_row.d;

    const int64_t s = load_vec<int64_t, false>(a.slots_at + (uint64_t(c) * a.chunk_tokens + t) * 8u);
    // the plane's base pointer is fetched while the slot is on its way
    const uint64_t layer = pin(uint64_t(layers.p[a.lp_base + lp]));
    const bool valid = uint64_t(s) < uint64_t(a.n_slots);  // negative wraps to huge
    if (s >= int64_t(a.n_slots)) store_vec<int32_t, false>(a.bad_flag_at, 1);
    const uint32_t su = valid ? uint32_t(s) : 0u;  // slot 0 is always inside the pages
    const uint32_t b = a.by_bs.div(su);
    const uint32_t o = su - b * a.by_bs.d;
    uint32_t run = 0, dv = w;
    if (a.runs_per_row > 1) {
        run = a.by_run.div(w);
        dv = w - run * a.by_run.d;
    }
    const uint64_t page = layer + uint64_t(int64_t(b) * a.block_stride + int64_t(o) * a.token_stride +
                                           int64_t(run) * a.run_stride + int64_t(dv) * VEC);
    const uint64_t st = a.staging_at + uint64_t(c) * a.chunk_stride + uint64_t(lp) * a.plane_bytes +
                        uint64_t(r) * VEC;
    if (GATHER) {
        V v = load_vec<V, NT_LD>(page);
        if (!valid) v = V(0);
        store_vec<V, NT_ST>(st, v);
    } else if (valid) {
        store_vec<V, NT_ST>(page, load_vec<V, NT_LD>(st));
    }
}

// HBM to HBM (pages <-> staging): one tile per workgroup, a very large grid.
template <int VEC, bool GATHER, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(kThreads) void move_rows(const KernelGeom g, const LaunchView view,
                                                      const LayerPtrs layers,
                                                      const int64_t *__restrict__ slot_mapping,
                                                      uint8_t *staging, int32_t *bad_flag,
                                                      uint32_t n_blocks_permuted, uint32_t xcd_shift) {
    const TileArgs a = fetch_args(g, view, slot_mapping, staging, bad_flag);
    uint32_t blk = blockIdx.x;
    if (blk < n_blocks_permuted) {
        // hardware deals consecutive workgroup ids to the 8 XCDs in turn; give each XCD
        // runs of 2^xcd_shift consecutive tiles instead of every eighth tile.  This is a
        // permutation inside every group of 8 << xcd_shift ids, and n_blocks_permuted is
        // a multiple of that, so the result stays below it.
        const uint32_t xcd = blk & 7u, local = blk >> 3;
        const uint32_t grp = local >> xcd_shift;
        blk = (((grp << 3) + xcd) << xcd_shift) + (local & ((1u << xcd_shift) - 1u));
    }
    move_tile<VEC, GATHER, NT_LD, NT_ST>(a, layers, blk);
}

// Across the host link (pages <-> pinned pool, no staging): the link, not HBM, sets the
// pace, and it runs best when few workgroups walk the host side in order.  Measured with a
// plain copy kernel on this part: 64 workgroups taking tiles in turn reach 57.6 GB/s
// reading host memory and 56.2 GB/s writing it (the runtime's own copies: 57.2 / 57.0),
// one tile per workgroup over thousands of workgroups 55.7 / 54.4.  The grid is fixed and
// every workgroup takes tiles blk, blk + gridDim.x, ... until the launch's n_blocks.
template <int VEC, bool GATHER, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(kThreads) void move_rows_paced(const KernelGeom g, const LaunchView view,
                                                            const LayerPtrs layers,
                                                            const int64_t *__restrict__ slot_mapping,
                                                            uint8_t *staging, int32_t *bad_flag,
                                                            uint32_t n_blocks) {
    const TileArgs a = fetch_args(g, view, slot_mapping, staging, bad_flag);
    const uint32_t step = pin(uint32_t(gridDim.x)), end = pin(n_blocks);
    for (uint32_t blk = blockIdx.x; blk < end; blk += step)
        move_tile<VEC, GATHER, NT_LD, NT_ST>(a, layers, blk);
}

// ---- scatter in the order of the destination ---------------------------------------------
// A launch that fills thousands of pages per plane (a long context, a batch of requests)
// finds many of its pages close together in memory, but the slot mapping names them in
// the order of the tokens, which is random in address.  Writes to DRAM are what suffers
// most from jumping around, so for such launches the rows are visited in ascending slot
// order, plane by plane: the writes then sweep each plane once, and the jumps move to the
// reads of the staging buffer.  The order is built on the device, without a sort: every
// slot number is an index into a table (one word per slot of a plane) that receives the
// token living there, and compacting the table yields (slot, token) pairs in slot order.

constexpr uint32_t kNoToken = 0xFFFFFFFFu;
constexpr int kSlotsPerThread = 8;
constexpr int kSlotsPerGroup = kThreads * kSlotsPerThread;

__global__ __launch_bounds__(kThreads) void order_clear(uint32_t *__restrict__ token_at, uint32_t n_slots) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n_slots) token_at[i] = kNoToken;
}

// token_at[slot] = token; slots outside the pages raise the flag, negative ones are left out
__global__ __launch_bounds__(kThreads) void order_mark(const int64_t *__restrict__ slot_mapping,
                                                       uint32_t n_tokens, uint32_t n_slots,
                                                       uint32_t *__restrict__ token_at, int32_t *bad_flag) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_tokens) return;
    const int64_t s = slot_mapping[i];
    if (s >= int64_t(n_slots)) *bad_flag = 1;
    else if (s >= 0) token_at[s] = i;
}

// exclusive prefix sum over the workgroup of one value per thread; *total = the sum
__device__ __forceinline__ uint32_t group_exclusive_scan(uint32_t v, uint32_t *lds, uint32_t *total) {
    const uint32_t t = threadIdx.x, n = blockDim.x;
    lds[t] = v;
    __syncthreads();
    for (uint32_t d = 1; d < n; d <<= 1) {
        const uint32_t add = t >= d ? lds[t - d] : 0u;
        __syncthreads();
        lds[t] += add;
        __syncthreads();
    }
    const uint32_t incl = lds[t];
    *total = lds[n - 1];
    __syncthreads();
    return incl - v;
}

__device__ __forceinline__ uint32_t occupied_in_my_slots(const uint32_t *token_at, uint32_t n_slots,
                                                         uint32_t first) {
    uint32_t cnt = 0;
    for (int k = 0; k < kSlotsPerThread; k++)
        cnt += (first + k < n_slots && token_at[first + k] != kNoToken) ? 1u : 0u;
    return cnt;
}

// counts[group] = occupied slots among the group's kSlotsPerGroup slots
__global__ __launch_bounds__(kThreads) void order_count(const uint32_t *__restrict__ token_at,
                                                        uint32_t n_slots, uint32_t *__restrict__ counts) {
    __shared__ uint32_t lds[kThreads];
    const uint32_t first = blockIdx.x * kSlotsPerGroup + threadIdx.x * kSlotsPerThread;
    uint32_t total;
    group_exclusive_scan(occupied_in_my_slots(token_at, n_slots, first), lds, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// one workgroup: counts[] becomes its exclusive prefix sum, *n_rows the grand total
__global__ __launch_bounds__(1024) void order_offsets(uint32_t *__restrict__ counts, uint32_t n_groups,
                                                      uint32_t *__restrict__ n_rows) {
    __shared__ uint32_t lds[1024];
    const uint32_t per = (n_groups + 1023u) / 1024u;
    const uint32_t lo = threadIdx.x * per, hi = lo + per < n_groups ? lo + per : n_groups;
    uint32_t sum = 0;
    for (uint32_t i = lo; i < hi; i++) sum += counts[i];
    uint32_t total;
    uint32_t run = group_exclusive_scan(sum, lds, &total);
    for (uint32_t i = lo; i < hi; i++) {
        const uint32_t c = counts[i];
        counts[i] = run;
        run += c;
    }
    if (threadIdx.x == 0) *n_rows = total;
}

// pairs[rank of the slot among the occupied ones] = (slot, token)
__global__ __launch_bounds__(kThreads) void order_emit(const uint32_t *__restrict__ token_at,
                                                       uint32_t n_slots, const uint32_t *__restrict__ offsets,
                                                       uint2 *__restrict__ pairs) {
    __shared__ uint32_t lds[kThreads];
    const uint32_t first = blockIdx.x * kSlotsPerGroup + threadIdx.x * kSlotsPerThread;
    uint32_t total;
    uint32_t at = offsets[blockIdx.x] +
                  group_exclusive_scan(occupied_in_my_slots(token_at, n_slots, first), lds, &total);
    for (int k = 0; k < kSlotsPerThread; k++) {
        if (first + k >= n_slots) break;
        const uint32_t tok = token_at[first + k];
        if (tok != kNoToken) pairs[at++] = make_uint2(first + k, tok);
    }
}

// The scatter itself.  The pairs are taken in groups of group_rows; workgroups are
// numbered group by group, inside a group plane by plane, inside a plane along the group's
// pairs: lane = vector w of the row of pair j.  So what is in flight at any moment is, in
// each of a few planes, a run of pages that are neighbours in address.  The launch is sized
// for the tokens of the call; the pairs may be fewer (tokens without a page), the rest of
// the grid retires.
template <int VEC, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(kThreads) void scatter_rows_ordered(const KernelGeom g, const LaunchView view,
                                                                 const LayerPtrs layers,
                                                                 const uint2 *__restrict__ pairs,
                                                                 const uint32_t *__restrict__ n_rows_at,
                                                                 const uint8_t *staging, FastDiv by_tiles_per_group,
                                                                 FastDiv by_chunk_tokens, uint32_t group_rows,
                                                                 uint32_t n_blocks_permuted, uint32_t xcd_shift) {
    typedef typename VecOf<VEC>::type V;
    const TileArgs a = fetch_args(g, view, nullptr, const_cast<uint8_t *>(staging), nullptr);
    const FastDiv by_tiles = pin(by_tiles_per_group), by_ct = pin(by_chunk_tokens);
    const uint64_t pairs_at = pin(uint64_t(pairs));
    const uint32_t n_rows = pin(*n_rows_at), rows = pin(group_rows);
    uint32_t blk = blockIdx.x;
    if (blk < n_blocks_permuted) {   // as in move_rows: runs of consecutive tiles per XCD
        const uint32_t xcd = blk & 7u, local = blk >> 3;
        const uint32_t grp = local >> xcd_shift;
        blk = (((grp << 3) + xcd) << xcd_shift) + (local & ((1u << xcd_shift) - 1u));
    }
    const uint32_t q = by_tiles.div(blk);
    const uint32_t tile = blk - q * by_tiles.d;
    const uint32_t grp = a.by_lp.div(q);
    const uint32_t lp = q - grp * a.by_lp.d;
    const uint32_t r = tile * kThreads + threadIdx.x;
    const uint32_t row = a.by_row.div(r);
    const uint32_t w = r - row * a.by_row.d;
    const uint32_t j = grp * rows + row;
    if (row >= rows || j >= n_rows) return;
    const typename VecOf<8>::type pr = load_vec<typename VecOf<8>::type, false>(pairs_at + uint64_t(j) * 8u);
    const uint64_t layer = pin(uint64_t(layers.p[a.lp_base + lp]));
    const uint32_t su = pr.x, tok = pr.y;
    const uint32_t c = by_ct.div(tok);
    const uint32_t t = tok - c * by_ct.d;
    const uint32_t b = a.by_bs.div(su);
    const uint32_t o = su - b * a.by_bs.d;
    uint32_t run = 0, dv = w;
    if (a.runs_per_row > 1) {
        run = a.by_run.div(w);
        dv = w - run * a.by_run.d;
    }
    const uint64_t page = layer + uint64_t(int64_t(b) * a.block_stride + int64_t(o) * a.token_stride +
                                           int64_t(run) * a.run_stride + int64_t(dv) * VEC);
    const uint64_t st = a.staging_at + uint64_t(c) * a.chunk_stride + uint64_t(lp) * a.plane_bytes +
                        (uint64_t(t) * a.by_row.d + w) * VEC;
    store_vec<V, NT_ST>(page, load_vec<V, NT_LD>(st));
}

__global__ __launch_bounds__(kThreads) void check_slots(const int64_t *__restrict__ slot_mapping,
                                                        uint64_t n, uint32_t n_slots,
                                                        int32_t *bad_flag) {
    uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    const uint64_t step = uint64_t(gridDim.x) * kThreads;
    bool bad = false;
    for (; i < n; i += step) bad |= slot_mapping[i] >= int64_t(n_slots);
    if (bad) *bad_flag = 1;
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Streaming copy, one 16-byte vector per lane, non-temporal both ways: the fastest of
// the plain-copy shapes measured on this part.
__global__ __launch_bounds__(kThreads) void copy_bytes(u32x4 *__restrict__ dst,
                                                       const u32x4 *__restrict__ src, uint64_t n_vec) {
    const uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n_vec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Plain copy of 4 KiB tiles in a given order, no slot mapping, no geometry: workgroup w
// copies tile src_order[w] of src to tile dst_order[w] of dst (a null order = w itself).
// Fed with the address stream of a gather or scatter launch it shows what the access
// pattern alone costs: the ceiling that launch can reach.  mode 1 only reads, mode 2 only
// writes (reads and writes react differently to scattered pages).
__global__ __launch_bounds__(kThreads) void copy_tiles(u32x4 *dst, const uint32_t *__restrict__ dst_order,
                                                       const u32x4 *src, const uint32_t *__restrict__ src_order,
                                                       uint32_t n_tiles, uint32_t mode, u32x4 *sink) {
    const uint32_t w = blockIdx.x;
    if (w >= n_tiles) return;
    const uint64_t s = (src_order ? uint64_t(src_order[w]) : uint64_t(w)) * kThreads + threadIdx.x;
    const uint64_t d = (dst_order ? uint64_t(dst_order[w]) : uint64_t(w)) * kThreads + threadIdx.x;
    if (mode == 0) {
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + s), dst + d);
    } else if (mode == 1) {
        const u32x4 v = __builtin_nontemporal_load(src + s);
        if (v.x == 0x9E3779B9u && v.y == 0x7F4A7C15u && v.z == 0xF39CC060u && v.w == 0x5CEDC834u) *sink = v;
    } else {
        const u32x4 v = {w, w, w, w};
        __builtin_nontemporal_store(v, dst + d);
    }
}

// Copy between device memory and the pinned pool, paced for the host link like
// move_rows_paced: a fixed, small grid whose workgroups take 4 KiB tiles in turn.  The
// bytes form `rows` rows of width_vec 16-byte vectors, src_pitch / dst_pitch bytes apart
// (one row per chunk; pitch == width gives a plain copy).
__global__ __launch_bounds__(kThreads) void copy_rect_paced(uint8_t *__restrict__ dst, uint64_t dst_pitch,
                                                            const uint8_t *__restrict__ src,
                                                            uint64_t src_pitch, uint64_t width_vec,
                                                            FastDiv by_tiles_per_row, uint32_t n_tiles) {
    const uint64_t dst_at = pin(uint64_t(dst)), src_at = pin(uint64_t(src));
    const uint64_t dp = pin(dst_pitch), sp = pin(src_pitch), wv = pin(width_vec);
    const FastDiv by_tpr = pin(by_tiles_per_row);
    const uint32_t step = pin(uint32_t(gridDim.x)), end = pin(n_tiles);
    for (uint32_t t = blockIdx.x; t < end; t += step) {
        const uint32_t row = by_tpr.div(t);
        const uint64_t v = uint64_t(t - row * by_tpr.d) * kThreads + threadIdx.x;
        if (v >= wv) continue;
        const u32x4 x = load_vec<u32x4, true>(src_at + uint64_t(row) * sp + v * 16u);
        store_vec<u32x4, true>(dst_at + uint64_t(row) * dp + v * 16u, x);
    }
}

// The same for pieces that lie in pool slots of any numbers (a fragmented pool): the row
// on the pool's side starts at slot[row] * pool_pitch.  One launch for all the pieces of a
// pipeline step, where the runtime would make one small copy per piece.
template <bool TO_POOL>
__global__ __launch_bounds__(kThreads) void copy_pieces_paced(uint8_t *__restrict__ pool, uint64_t pool_pitch,
                                                              uint8_t *__restrict__ staging, uint64_t stage_pitch,
                                                              uint64_t width_vec, FastDiv by_tiles_per_row,
                                                              uint32_t n_tiles, PieceSlots slots) {
    const uint64_t pool_at = pin(uint64_t(pool)), stage_at = pin(uint64_t(staging));
    const uint64_t pp = pin(pool_pitch), sp = pin(stage_pitch), wv = pin(width_vec);
    const FastDiv by_tpr = pin(by_tiles_per_row);
    const uint32_t step = pin(uint32_t(gridDim.x)), end = pin(n_tiles);
    for (uint32_t t = blockIdx.x; t < end; t += step) {
        const uint32_t row = by_tpr.div(t);
        const uint64_t v = uint64_t(t - row * by_tpr.d) * kThreads + threadIdx.x;
        if (v >= wv) continue;
        const uint64_t in_pool = pool_at + uint64_t(uint32_t(slots.slot[row])) * pp + v * 16u;
        const uint64_t in_stage = stage_at + uint64_t(row) * sp + v * 16u;
        const u32x4 x = load_vec<u32x4, true>(TO_POOL ? in_stage : in_pool);
        store_vec<u32x4, true>(TO_POOL ? in_pool : in_stage, x);
    }
}

__global__ __launch_bounds__(kThreads) void fill_bytes(uint8_t *dst, uint8_t value, uint64_t n) {
    const uint64_t step = uint64_t(gridDim.x) * kThreads;
    for (uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x; i < n; i += step)
        dst[i] = value;
}

template <int VEC, bool GATHER>
hipError_t launch_move_v(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                         const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                         uint8_t *staging, int32_t *bad_flag, hipStream_t stream, hipEvent_t start,
                         hipEvent_t stop) {
    const uint32_t n_blocks = n_chunks * v.by_n_lp.d * g.by_tiles_per_plane.d;
    if (n_blocks == 0) return hipSuccess;
    uint32_t shift = 0, permuted = 0;
    if (s.xcd_run > 0) {
        while ((2u << shift) <= s.xcd_run) shift++;                      // floor(log2(xcd_run))
        permuted = n_blocks & ~((8u << shift) - 1u);                     // the tail keeps its order
    }
    dim3 grid(n_blocks), block(kThreads);
    if (s.paced_groups > 0) {
        // blk + step must not wrap: n_blocks < 2^24 (max_chunks_per_launch) and the grid is small
        grid = dim3(std::min(n_blocks, s.paced_groups));
#define LMC_GO(LD, ST)                                                                                \
    hipExtLaunchKernelGGL((move_rows_paced<VEC, GATHER, LD, ST>), grid, block, 0, stream, start, stop, \
                          0, g, v, layers, slot_mapping, staging, bad_flag, n_blocks)
        if (s.nt_load && s.nt_store) LMC_GO(true, true);
        else if (s.nt_load) LMC_GO(true, false);
        else if (s.nt_store) LMC_GO(false, true);
        else LMC_GO(false, false);
#undef LMC_GO
        return hipGetLastError();
    }
#define LMC_GO(LD, ST)                                                                          \
    hipExtLaunchKernelGGL((move_rows<VEC, GATHER, LD, ST>), grid, block, 0, stream, start, stop, \
                          0, g, v, layers, slot_mapping, staging, bad_flag, permuted, shift)
    if (s.nt_load && s.nt_store) LMC_GO(true, true);
    else if (s.nt_load) LMC_GO(true, false);
    else if (s.nt_store) LMC_GO(false, true);
    else LMC_GO(false, false);
#undef LMC_GO
    return hipGetLastError();
}

template <bool GATHER>
hipError_t launch_move(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                       const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                       uint8_t *staging, int32_t *bad_flag, hipStream_t stream, hipEvent_t start,
                       hipEvent_t stop) {
    switch (g.vec) {
        case 16: return launch_move_v<16, GATHER>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream, start, stop);
        case 8: return launch_move_v<8, GATHER>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream, start, stop);
        case 4: return launch_move_v<4, GATHER>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream, start, stop);
        case 2: return launch_move_v<2, GATHER>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream, start, stop);
        case 1: return launch_move_v<1, GATHER>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream, start, stop);
    }
    return hipErrorInvalidValue;
}

}  // namespace

FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    if (d <= 1) {
        f.mul = 0;
        f.shift = 0;
        return f;
    }
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) l++;
    f.mul = uint32_t((uint64_t(1) << (31 + l)) / d + 1);
    f.shift = l - 1;
    return f;
}

uint32_t max_chunks_per_launch(const KernelGeom &g, const LaunchView &v) {
    // the workgroup index must stay below 2^31 for the fast division, and a launch's
    // thread count (workgroups x 256) below 2^32, the stricter of the two: 2^24 - 1
    // workgroups, 64 GiB at 4 KiB tiles
    return uint32_t(0x00FFFFFFu / (uint64_t(v.by_n_lp.d) * g.by_tiles_per_plane.d));
}

LaunchView bulk_view(const KernelGeom &g) {
    LaunchView v;
    v.by_n_lp = make_fastdiv(g.n_layer_planes);
    v.lp_base = 0;
    v.chunk_stride = g.chunk_bytes;
    return v;
}

LaunchView layer_view(const KernelGeom &g, uint32_t planes_per_layer, uint32_t first_layer,
                      uint32_t n_layers) {
    LaunchView v;
    v.by_n_lp = make_fastdiv(n_layers * planes_per_layer);
    v.lp_base = first_layer * planes_per_layer;
    v.chunk_stride = uint64_t(n_layers) * planes_per_layer * g.plane_bytes;
    return v;
}

hipError_t launch_gather(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                         const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                         uint8_t *staging, int32_t *bad_flag, hipStream_t stream, hipEvent_t start,
                         hipEvent_t stop) {
    return launch_move<true>(g, v, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream,
                             start, stop);
}

hipError_t launch_scatter(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                          const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_chunks,
                          const uint8_t *staging, int32_t *bad_flag, hipStream_t stream,
                          hipEvent_t start, hipEvent_t stop) {
    return launch_move<false>(g, v, s, layers, slot_mapping, n_chunks,
                              const_cast<uint8_t *>(staging), bad_flag, stream, start, stop);
}

uint64_t order_table_words(const KernelGeom &g) { return g.n_slots; }
uint64_t order_count_words(const KernelGeom &g) { return (uint64_t(g.n_slots) + kSlotsPerGroup - 1) / kSlotsPerGroup; }

// rows per group: the launch's choice, rounded so that a group is whole tiles where it can be
static uint32_t ordered_group_rows(const KernelGeom &g, const LaunchShape &s, uint64_t n_tokens) {
    uint64_t rows = s.ordered_group_rows == 0 ? n_tokens : std::min<uint64_t>(s.ordered_group_rows, n_tokens);
    return uint32_t(std::max<uint64_t>(rows, 1));
}

static uint64_t ordered_blocks(const KernelGeom &g, const LaunchView &v, uint64_t n_tokens, uint64_t rows) {
    const uint64_t tiles_per_group = (rows * g.by_vec_per_row.d + kThreads - 1) / kThreads;
    const uint64_t groups = (n_tokens + rows - 1) / rows;
    return groups * v.by_n_lp.d * tiles_per_group;
}

bool ordered_scatter_fits(const KernelGeom &g, const LaunchView &v, const LaunchShape &s, uint64_t n_tokens) {
    if (n_tokens == 0 || n_tokens >= (uint64_t(1) << 31) || g.n_slots > kMaxOrderedSlots) return false;
    const uint64_t rows = ordered_group_rows(g, s, n_tokens);
    if (rows * g.by_vec_per_row.d >= (uint64_t(1) << 31)) return false;   // lanes of one group and plane
    return ordered_blocks(g, v, n_tokens, rows) <= 0x00FFFFFFu;           // as max_chunks_per_launch
}

template <int VEC>
static hipError_t launch_scatter_ordered_v(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                                           const LayerPtrs &layers, uint32_t n_tokens, const OrderScratch &o,
                                           const uint8_t *staging, hipStream_t stream, hipEvent_t start,
                                           hipEvent_t stop) {
    const uint32_t rows = ordered_group_rows(g, s, n_tokens);
    const uint32_t tiles_per_group = uint32_t((uint64_t(rows) * g.by_vec_per_row.d + kThreads - 1) / kThreads);
    const uint32_t n_blocks = uint32_t(ordered_blocks(g, v, n_tokens, rows));
    uint32_t shift = 0, permuted = 0;
    if (s.xcd_run > 0) {
        while ((2u << shift) <= s.xcd_run) shift++;
        permuted = n_blocks & ~((8u << shift) - 1u);
    }
    const FastDiv by_tiles = make_fastdiv(tiles_per_group), by_ct = make_fastdiv(g.chunk_tokens);
    dim3 grid(n_blocks), block(kThreads);
#define LMC_GO(LD, ST)                                                                                 \
    hipExtLaunchKernelGGL((scatter_rows_ordered<VEC, LD, ST>), grid, block, 0, stream, start, stop, 0, g, \
                          v, layers, o.pairs, o.n_rows, staging, by_tiles, by_ct, rows, permuted, shift)
    if (s.nt_load && s.nt_store) LMC_GO(true, true);
    else if (s.nt_load) LMC_GO(true, false);
    else if (s.nt_store) LMC_GO(false, true);
    else LMC_GO(false, false);
#undef LMC_GO
    return hipGetLastError();
}

hipError_t launch_scatter_ordered(const KernelGeom &g, const LaunchView &v, const LaunchShape &s,
                                  const LayerPtrs &layers, const int64_t *slot_mapping, uint32_t n_tokens,
                                  const OrderScratch &o, const uint8_t *staging, int32_t *bad_flag,
                                  hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
    if (n_tokens == 0) return hipSuccess;
    const uint32_t n_slots = g.n_slots;
    const uint32_t n_groups = uint32_t(order_count_words(g));
    const dim3 block(kThreads);
    hipLaunchKernelGGL(order_clear, dim3((n_slots + kThreads - 1) / kThreads), block, 0, stream, o.token_at, n_slots);
    hipLaunchKernelGGL(order_mark, dim3((n_tokens + kThreads - 1) / kThreads), block, 0, stream, slot_mapping,
                       n_tokens, n_slots, o.token_at, bad_flag);
    hipLaunchKernelGGL(order_count, dim3(n_groups), block, 0, stream, o.token_at, n_slots, o.counts);
    hipLaunchKernelGGL(order_offsets, dim3(1), dim3(1024), 0, stream, o.counts, n_groups, o.n_rows);
    hipLaunchKernelGGL(order_emit, dim3(n_groups), block, 0, stream, o.token_at, n_slots, o.counts, o.pairs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (g.vec) {
        case 16: return launch_scatter_ordered_v<16>(g, v, s, layers, n_tokens, o, staging, stream, start, stop);
        case 8: return launch_scatter_ordered_v<8>(g, v, s, layers, n_tokens, o, staging, stream, start, stop);
        case 4: return launch_scatter_ordered_v<4>(g, v, s, layers, n_tokens, o, staging, stream, start, stop);
        case 2: return launch_scatter_ordered_v<2>(g, v, s, layers, n_tokens, o, staging, stream, start, stop);
        case 1: return launch_scatter_ordered_v<1>(g, v, s, layers, n_tokens, o, staging, stream, start, stop);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_check_slots(const int64_t *slot_mapping, uint64_t n, uint32_t n_slots,
                              int32_t *bad_flag, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(check_slots, dim3(uint32_t(blocks)), dim3(kThreads), 0, stream, slot_mapping,
                       n, n_slots, bad_flag);
    return hipGetLastError();
}

hipError_t launch_copy(uint8_t *dst, const uint8_t *src, uint64_t nbytes, hipStream_t stream) {
    const uint64_t n_vec = nbytes / 16;
    const uint64_t per_launch = uint64_t(0x00FFFFFFu) * kThreads;   // a launch's threads stay below 2^32
    for (uint64_t v0 = 0; v0 < n_vec; v0 += per_launch) {
        const uint64_t n = n_vec - v0 < per_launch ? n_vec - v0 : per_launch;
        hipLaunchKernelGGL(copy_bytes, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads),
                           0, stream, reinterpret_cast<u32x4 *>(dst) + v0,
                           reinterpret_cast<const u32x4 *>(src) + v0, n);
    }
    return hipGetLastError();
}

hipError_t launch_copy_tiles(uint8_t *dst, const uint32_t *dst_order, const uint8_t *src,
                             const uint32_t *src_order, uint32_t n_tiles, uint32_t mode, uint8_t *sink,
                             hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    if (n_tiles > 0x7FFFFFFFu || mode > 2) return hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_tiles, dim3(n_tiles), dim3(kThreads), 0, stream, reinterpret_cast<u32x4 *>(dst), dst_order,
                       reinterpret_cast<const u32x4 *>(src), src_order, n_tiles, mode, reinterpret_cast<u32x4 *>(sink));
    return hipGetLastError();
}

hipError_t launch_copy_rect(uint8_t *dst, uint64_t dst_pitch, const uint8_t *src, uint64_t src_pitch,
                            uint64_t width, uint64_t rows, uint32_t groups, hipStream_t stream) {
    if (width == 0 || rows == 0) return hipSuccess;
    if ((width % 16) != 0 || (dst_pitch % 16) != 0 || (src_pitch % 16) != 0 || groups == 0 ||
        (reinterpret_cast<uintptr_t>(dst) % 16) != 0 || (reinterpret_cast<uintptr_t>(src) % 16) != 0)
        return hipErrorInvalidValue;
    const uint64_t width_vec = width / 16;
    const uint64_t tiles_per_row = (width_vec + kThreads - 1) / kThreads;
    if (tiles_per_row >= (uint64_t(1) << 24)) return hipErrorInvalidValue;   // 64 GiB rows: not a chunk
    // the tile index is 32-bit and stays below 2^24, so t + grid never wraps and FastDiv is exact
    const uint64_t rows_per_launch = std::max<uint64_t>(1, uint64_t(0x00FFFFFFu) / tiles_per_row);
    for (uint64_t r0 = 0; r0 < rows; r0 += rows_per_launch) {
        const uint64_t n = std::min(rows - r0, rows_per_launch);
        const uint32_t n_tiles = uint32_t(n * tiles_per_row);
        hipLaunchKernelGGL(copy_rect_paced, dim3(std::min(n_tiles, groups)), dim3(kThreads), 0, stream,
                           dst + r0 * dst_pitch, dst_pitch, src + r0 * src_pitch, src_pitch, width_vec,
                           make_fastdiv(uint32_t(tiles_per_row)), n_tiles);
    }
    return hipGetLastError();
}

hipError_t launch_copy_pieces(uint8_t *pool, uint64_t pool_pitch, uint8_t *staging, uint64_t stage_pitch,
                              uint64_t width, const PieceSlots &slots, uint32_t n_pieces, bool to_pool,
                              uint32_t groups, hipStream_t stream) {
    if (width == 0 || n_pieces == 0) return hipSuccess;
    if ((width % 16) != 0 || (pool_pitch % 16) != 0 || (stage_pitch % 16) != 0 || groups == 0 ||
        n_pieces > uint32_t(kMaxPieces) || (reinterpret_cast<uintptr_t>(pool) % 16) != 0 ||
        (reinterpret_cast<uintptr_t>(staging) % 16) != 0)
        return hipErrorInvalidValue;
    for (uint32_t i = 0; i < n_pieces; i++)
        if (slots.slot[i] < 0) return hipErrorInvalidValue;
    const uint64_t width_vec = width / 16;
    const uint64_t tiles_per_row = (width_vec + kThreads - 1) / kThreads;
    // the tile index is 32-bit and stays below 2^24, so t + grid never wraps and FastDiv is exact
    if (tiles_per_row * n_pieces >= (uint64_t(1) << 24)) return hipErrorInvalidValue;
    const uint32_t n_tiles = uint32_t(tiles_per_row * n_pieces);
    const dim3 grid(std::min(n_tiles, groups)), block(kThreads);
    if (to_pool)
        hipLaunchKernelGGL(copy_pieces_paced<true>, grid, block, 0, stream, pool, pool_pitch, staging, stage_pitch,
                           width_vec, make_fastdiv(uint32_t(tiles_per_row)), n_tiles, slots);
    else
        hipLaunchKernelGGL(copy_pieces_paced<false>, grid, block, 0, stream, pool, pool_pitch, staging, stage_pitch,
                           width_vec, make_fastdiv(uint32_t(tiles_per_row)), n_tiles, slots);
    return hipGetLastError();
}

hipError_t launch_fill(uint8_t *dst, uint8_t value, uint64_t nbytes, hipStream_t stream) {
    if (nbytes == 0) return hipSuccess;
    uint64_t blocks = (nbytes + kThreads - 1) / kThreads;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_bytes, dim3(uint32_t(blocks)), dim3(kThreads), 0, stream, dst, value,
                       nbytes);
    return hipGetLastError();
}

}  // namespace lmc
