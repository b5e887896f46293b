// Device kernels of liblmc for gfx950 (MI355X): the paged-KV gather (store direction)
// and scatter (load direction) that the paper's section 5.1 places between the
// engine's pages and the contiguous streaming GPU buffer, plus small helpers.
//
// Both kernels are pure byte movement and HBM-bound.  Work split:
//   - a lane owns one `vec`-byte vector of one token's row: the pair (token t, vector w)
//     of chunk c.  It reads the token's slot once, turns it into a byte offset inside
//     a layer-plane once, and then walks the layer-planes of its workgroup's range:
//     per step one scalar load of the plane's base pointer, one 64-bit add, one
//     16-byte load and one 16-byte store.  The slot lookup and the division by the
//     block size are amortised over every layer and plane.
//   - consecutive lanes own consecutive vectors of a row and then the next token, so a
//     wavefront's access is 1 KiB contiguous on the chunk side and, on the page side,
//     contiguous for as long as the row (or head run) and the page go on.
//   - kUnroll independent loads are issued before the first store, which is what keeps
//     enough bytes in flight per CU to cover HBM latency.
//   - grid = (pairs / 256, layer-plane groups): the second dimension exists so that a
//     launch over one chunk still gives several workgroups per CU.
#include "lmc_kernels.hpp"

namespace lmc {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;

template <int N> struct VecOf;
template <> struct VecOf<16> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef unsigned int type; };
template <> struct VecOf<2> { typedef unsigned short type; };
template <> struct VecOf<1> { typedef unsigned char type; };

template <typename V, bool NT> __device__ __forceinline__ V load_vec(const uint8_t *p) {
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
    return *reinterpret_cast<const V *>(p);
}
template <typename V, bool NT> __device__ __forceinline__ void store_vec(uint8_t *p, V v) {
    if (NT) __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
    else *reinterpret_cast<V *>(p) = v;
}

// One pass of the path's copy in either direction.
//   GATHER: chunk[c][lp][t][w] = valid ? page(lp, slot)[w] : 0
//   else  : if (valid) page(lp, slot)[w] = chunk[c][lp][t][w]
template <int VEC, bool GATHER, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(kThreads) void move_rows(const KernelGeom g, const LayerPtrs layers,
                                                      const int64_t *__restrict__ slot_mapping,
                                                      uint32_t n_pairs, uint8_t *staging,
                                                      int32_t *bad_flag, uint32_t lp_per_block) {
    typedef typename VecOf<VEC>::type V;
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_pairs) return;
    const uint32_t c = i / g.pairs_per_chunk;
    const uint32_t r = i - c * g.pairs_per_chunk;  // vector index inside one layer-plane of the chunk
    const uint32_t t = r / g.vec_per_row;
    const uint32_t w = r - t * g.vec_per_row;

    const int64_t s = slot_mapping[uint64_t(c) * g.chunk_tokens + t];
    const bool valid = uint64_t(s) < uint64_t(g.n_slots);  // negative wraps to huge
    if (s >= int64_t(g.n_slots)) *bad_flag = 1;
    const uint32_t su = valid ? uint32_t(s) : 0u;  // slot 0 is always inside the pages
    uint32_t b, o;
    if (g.block_shift >= 0) {
        b = su >> g.block_shift;
        o = su & (g.block_size - 1u);
    } else {
        b = su / g.block_size;
        o = su - b * g.block_size;
    }
    uint32_t run = 0, dv = w;
    if (g.runs_per_row > 1) {
        run = w / g.vec_per_run;
        dv = w - run * g.vec_per_run;
    }
    const int64_t page_off = int64_t(b) * g.block_stride + int64_t(o) * g.token_stride +
                             int64_t(run) * g.run_stride + int64_t(dv) * VEC;

    const uint32_t lp0 = blockIdx.y * lp_per_block;
    const uint32_t lp1 = min(lp0 + lp_per_block, g.n_layer_planes);
    uint8_t *st = staging + uint64_t(c) * g.chunk_bytes + uint64_t(lp0) * g.row_stride_lp +
                  uint64_t(r) * VEC;

    uint32_t lp = lp0;
    for (; lp + kUnroll <= lp1; lp += kUnroll) {
        V v[kUnroll];
        if (GATHER) {
#pragma unroll
            for (int u = 0; u < kUnroll; u++)
                v[u] = load_vec<V, NT_LD>(layers.p[lp + u] + page_off);
#pragma unroll
            for (int u = 0; u < kUnroll; u++) {
                if (!valid) v[u] = V(0);
                store_vec<V, NT_ST>(st + uint64_t(u) * g.row_stride_lp, v[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; u++)
                v[u] = load_vec<V, NT_LD>(st + uint64_t(u) * g.row_stride_lp);
            if (valid) {
#pragma unroll
                for (int u = 0; u < kUnroll; u++)
                    store_vec<V, NT_ST>(layers.p[lp + u] + page_off, v[u]);
            }
        }
        st += uint64_t(kUnroll) * g.row_stride_lp;
    }
    for (; lp < lp1; lp++) {
        if (GATHER) {
            V v = load_vec<V, NT_LD>(layers.p[lp] + page_off);
            if (!valid) v = V(0);
            store_vec<V, NT_ST>(st, v);
        } else if (valid) {
            store_vec<V, NT_ST>(layers.p[lp] + page_off, load_vec<V, NT_LD>(st));
        }
        st += g.row_stride_lp;
    }
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

// Streaming copy: 4 independent 16-byte loads per lane per step, grid-stride.
__global__ __launch_bounds__(kThreads) void copy_bytes(u32x4 *__restrict__ dst,
                                                       const u32x4 *__restrict__ src, uint64_t n_vec) {
    const uint64_t step = uint64_t(gridDim.x) * kThreads;
    uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    for (; i + 3 * step < n_vec; i += 4 * step) {
        u32x4 a = __builtin_nontemporal_load(src + i);
        u32x4 b = __builtin_nontemporal_load(src + i + step);
        u32x4 c = __builtin_nontemporal_load(src + i + 2 * step);
        u32x4 d = __builtin_nontemporal_load(src + i + 3 * step);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + step);
        __builtin_nontemporal_store(c, dst + i + 2 * step);
        __builtin_nontemporal_store(d, dst + i + 3 * step);
    }
    for (; i < n_vec; i += step) dst[i] = src[i];
}

__global__ __launch_bounds__(kThreads) void fill_bytes(uint8_t *dst, uint8_t value, uint64_t n) {
    const uint64_t step = uint64_t(gridDim.x) * kThreads;
    for (uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x; i < n; i += step)
        dst[i] = value;
}

template <int VEC, bool GATHER>
hipError_t launch_move_v(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                         const int64_t *slot_mapping, uint32_t n_chunks, uint8_t *staging,
                         int32_t *bad_flag, hipStream_t stream) {
    const uint32_t n_pairs = n_chunks * g.pairs_per_chunk;
    const uint32_t lpb = s.lp_per_block < 1 ? 1 : s.lp_per_block;
    dim3 grid((n_pairs + kThreads - 1) / kThreads, (g.n_layer_planes + lpb - 1) / lpb);
    dim3 block(kThreads);
    if (grid.x == 0) return hipSuccess;
#define LMC_GO(LD, ST)                                                                          \
    hipLaunchKernelGGL((move_rows<VEC, GATHER, LD, ST>), grid, block, 0, stream, g, layers,     \
                       slot_mapping, n_pairs, staging, bad_flag, lpb)
    if (s.nt_load && s.nt_store) LMC_GO(true, true);
    else if (s.nt_load) LMC_GO(true, false);
    else if (s.nt_store) LMC_GO(false, true);
    else LMC_GO(false, false);
#undef LMC_GO
    return hipGetLastError();
}

template <bool GATHER>
hipError_t launch_move(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                       const int64_t *slot_mapping, uint32_t n_chunks, uint8_t *staging,
                       int32_t *bad_flag, hipStream_t stream) {
    switch (g.vec) {
        case 16: return launch_move_v<16, GATHER>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
        case 8: return launch_move_v<8, GATHER>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
        case 4: return launch_move_v<4, GATHER>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
        case 2: return launch_move_v<2, GATHER>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
        case 1: return launch_move_v<1, GATHER>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

uint32_t max_chunks_per_launch(const KernelGeom &g) {
    // the pair index and the x grid dimension are 32-bit
    return uint32_t(0x7FFFFFFFu / g.pairs_per_chunk);
}

hipError_t launch_gather(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                         const int64_t *slot_mapping, uint32_t n_chunks, uint8_t *staging,
                         int32_t *bad_flag, hipStream_t stream) {
    return launch_move<true>(g, s, layers, slot_mapping, n_chunks, staging, bad_flag, stream);
}

hipError_t launch_scatter(const KernelGeom &g, const LaunchShape &s, const LayerPtrs &layers,
                          const int64_t *slot_mapping, uint32_t n_chunks, const uint8_t *staging,
                          int32_t *bad_flag, hipStream_t stream) {
    return launch_move<false>(g, s, layers, slot_mapping, n_chunks, const_cast<uint8_t *>(staging),
                              bad_flag, stream);
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
    if (n_vec == 0) return hipSuccess;
    uint64_t blocks = (n_vec + kThreads * 4 - 1) / (kThreads * 4);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(copy_bytes, dim3(uint32_t(blocks)), dim3(kThreads), 0, stream,
                       reinterpret_cast<u32x4 *>(dst), reinterpret_cast<const u32x4 *>(src), n_vec);
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
