// Ablation variants of Bitpack / Bitunpack (Section III, Algorithms 2 and 5 of
// arXiv 2004.02297) for gfx950.  They produce the same bytes as the production
// kernels and exist only to measure what each design choice buys:
//   kNaive     one thread per weight, byte accesses on the stream side (the
//              direct GPU rendering of the per-weight loops of Algorithms 2/5);
//   kVecDirect 128-bit loads of four weights per lane, top bytes kept in
//              registers, then one 4r-byte store per lane straight to the
//              stream (no LDS pass): coalesced, but 4/8/12-byte wide;
//   kPerLayer  the production kernel, launched once per layer instead of once
//              for all layers.
// kVecDirect needs every layer's stream offset and element offset to be a
// multiple of 4 (true for all CNN-shaped sets); the entry point checks this.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_launch.h"
#include "adt_tables.h"
#include "adt_tile_ops.h"

namespace adt {


__device__ __forceinline__ int find_layer(const uint32_t *tile_off, int n_layers, uint32_t block) {
    int lo = 0, hi = n_layers;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_off[mid] <= block) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kBlock) void naive_pack_kernel(const AblationArgs a) {
    const int l = find_layer(a.tile_off, a.n_layers, blockIdx.x);
    const int64_t i = (int64_t)(blockIdx.x - a.tile_off[l]) * kNaiveTile + threadIdx.x;
    const int64_t n = a.elem_off[l + 1] - a.elem_off[l];
    if (i >= n) return;
    const int r = a.rbytes[l];
    const uint32_t word = a.weights[a.elem_off[l] + i];
    uint8_t *dst = a.packed + a.pack_off[l] + i * r;
    for (int k = 0; k < r; ++k) dst[k] = (uint8_t)(word >> (8 * (4 - r + k)));
}

__global__ __launch_bounds__(kBlock) void naive_unpack_kernel(const AblationArgs a) {
    const int l = find_layer(a.tile_off, a.n_layers, blockIdx.x);
    const int64_t i = (int64_t)(blockIdx.x - a.tile_off[l]) * kNaiveTile + threadIdx.x;
    const int64_t n = a.elem_off[l + 1] - a.elem_off[l];
    if (i >= n) return;
    const int r = a.rbytes[l];
    const uint8_t *src = a.packed + a.pack_off[l] + i * r;
    uint32_t q = 0;
    for (int k = 0; k < r; ++k) q |= (uint32_t)src[k] << (8 * k);
    const_cast<uint32_t *>(a.weights)[a.elem_off[l] + i] = q << (8 * (4 - r));
}

template <int R>
__device__ __forceinline__ void vec_direct_store(uint8_t *dst, const u32x4 v) {
    uint32_t d[4];
    keep_top_bytes<R>(v, d);
    uint32_t *p = (uint32_t *)dst;        // 4-byte aligned by the entry point's check
#pragma unroll
    for (int t = 0; t < R; ++t) p[t] = d[t];
}

__global__ __launch_bounds__(kBlock) void vec_direct_pack_kernel(const AblationArgs a) {
    const int l = find_layer(a.tile_off, a.n_layers, blockIdx.x);
    const int64_t e0 = (int64_t)(blockIdx.x - a.tile_off[l]) * kVecTile + 4 * (int64_t)threadIdx.x;
    const int64_t n = a.elem_off[l + 1] - a.elem_off[l];
    if (e0 >= n) return;
    const int r = a.rbytes[l];
    const uint32_t *src = a.weights + a.elem_off[l] + e0;
    uint8_t *dst = a.packed + a.pack_off[l] + e0 * r;
    if (e0 + 4 <= n) {
        const u32x4 v = *(const u32x4_a4 *)src;
        switch (r) {
            case 1: vec_direct_store<1>(dst, v); break;
            case 2: vec_direct_store<2>(dst, v); break;
            case 3: vec_direct_store<3>(dst, v); break;
            default: vec_direct_store<4>(dst, v); break;
        }
    } else {
        for (int64_t i = e0; i < n; ++i) {
            const uint32_t word = src[i - e0];
            for (int k = 0; k < r; ++k) dst[(i - e0) * r + k] = (uint8_t)(word >> (8 * (4 - r + k)));
        }
    }
}

hipError_t launch_ablation(int which, const AblationArgs &a, uint32_t n_tiles, hipStream_t s) {
    switch (which) {
        case 0: naive_pack_kernel<<<dim3(n_tiles), dim3(kBlock), 0, s>>>(a); break;
        case 1: naive_unpack_kernel<<<dim3(n_tiles), dim3(kBlock), 0, s>>>(a); break;
        default: vec_direct_pack_kernel<<<dim3(n_tiles), dim3(kBlock), 0, s>>>(a); break;
    }
    return hipGetLastError();
}

}  // namespace adt
