// Per-layer statistics of AWP for gfx950 (Section II of arXiv 2004.02297:
// the l2-norm of all weights of a layer, taken every batch).
//
// Two launches for all layers together:
//   1. partial kernel: the grid is the concatenation of every layer's tiles
//      of 8192 weights.  A lane issues 128-bit loads (nontemporal: each
//      weight is read once), squares in double
//      precision (the square of a binary32 value is exact in binary64) and
//      keeps four running sums; a wave combines its lanes with xor-shuffles,
//      the block combines its four waves through LDS, and one partial
//      {sum of squares, largest magnitude} per tile goes to scratch memory.
//   2. final kernel: one block of 1024 threads per layer adds that layer's
//      partials in a fixed order and writes {sum, sqrt(sum), max |w|}.
// No atomics: the order of every addition is fixed by the indices alone, so
// the result is bit-identical from run to run.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_launch.h"
#include "adt_tables.h"
#include "awp_partials.h"

namespace adt {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

__device__ __forceinline__ void block_combine(double sum, uint32_t mag, double *out_sum,
                                              uint32_t *out_mag) {
    __shared__ double wsum[kWavesPerBlock];
    __shared__ uint32_t wmag[kWavesPerBlock];
    sum = wave_sum(sum);
    mag = wave_max(mag);
    const int wave = (int)(threadIdx.x >> 6);
    if ((threadIdx.x & 63) == 0) {
        wsum[wave] = sum;
        wmag[wave] = mag;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        *out_sum = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
        uint32_t m = wmag[0];
#pragma unroll
        for (int i = 1; i < kWavesPerBlock; ++i) m = wmag[i] > m ? wmag[i] : m;
        *out_mag = m;
    }
}

template <bool INLINE>
__global__ __launch_bounds__(kBlock) void stats_partial_kernel(const StatsArgs a) {
    const uint32_t *tile_off = INLINE ? a.inl.tile_off : a.dev_tile_off;
    const int64_t *elem_off = INLINE ? a.inl.elem_off : a.dev_elem_off;
    const uint32_t block = blockIdx.x;
    int lo = 0, hi = a.n_layers;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (table_load(tile_off, mid) <= block) lo = mid; else hi = mid;
    }
    const int64_t e_begin = table_load(elem_off, lo);
    const int64_t first = (int64_t)(block - table_load(tile_off, lo)) * kStatsTile;
    const int64_t left = (table_load(elem_off, lo + 1) - e_begin) - first;   // > 0 by construction
    const int len = left < kStatsTile ? (int)left : kStatsTile;
    const uint32_t *src = a.weights + e_begin + first;
    const int tid = (int)threadIdx.x;

    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    uint32_t mag = 0u;
    if (len == kStatsTile) {
        u32x4 v[kStatsLoadsPerLane];        // all of a lane's loads are in flight together
#pragma unroll
        for (int j = 0; j < kStatsLoadsPerLane; ++j)
            v[j] = __builtin_nontemporal_load((const u32x4_a4 *)(src + 4 * (j * kBlock + tid)));
#pragma unroll
        for (int j = 0; j < kStatsLoadsPerLane; ++j) {
            square_add(v[j].x, acc0, mag);
            square_add(v[j].y, acc1, mag);
            square_add(v[j].z, acc2, mag);
            square_add(v[j].w, acc3, mag);
        }
    } else {
        for (int i = 0; i < kStatsLoadsPerLane; ++i) {
            const int e0 = 4 * (i * kBlock + tid);
            if (e0 + 4 <= len) {
                const u32x4 v = __builtin_nontemporal_load((const u32x4_a4 *)(src + e0));
                square_add(v.x, acc0, mag);
                square_add(v.y, acc1, mag);
                square_add(v.z, acc2, mag);
                square_add(v.w, acc3, mag);
            } else {
                if (e0 < len) square_add(src[e0], acc0, mag);
                if (e0 + 1 < len) square_add(src[e0 + 1], acc1, mag);
                if (e0 + 2 < len) square_add(src[e0 + 2], acc2, mag);
            }
        }
    }
    block_combine((acc0 + acc1) + (acc2 + acc3), mag, &a.partial_sumsq[block],
                  &a.partial_absmax[block]);
}

template <bool INLINE>
__global__ __launch_bounds__(kFinalBlock) void stats_final_kernel(const StatsFinalArgs a) {
    const uint32_t *tile_off = INLINE ? a.inl_tile_off : a.dev_tile_off;
    const int layer = (int)blockIdx.x;
    double tot;
    uint32_t tm;
    reduce_partials(a.partial_sumsq, a.partial_absmax, tile_off[layer], tile_off[layer + 1], tot, tm);
    if (threadIdx.x == 0) {
        double *o = a.stats_out + (int64_t)layer * 3;
        o[0] = tot;
        o[1] = sqrt(tot);
        o[2] = (double)__uint_as_float(tm);   // NaN bits stay NaN
    }
}

hipError_t launch_stats(const StatsArgs &a, const StatsFinalArgs &f, uint32_t n_tiles,
                        bool inline_table, uint32_t extra_lds, hipStream_t stream) {
    if (n_tiles > 0) {
        hipError_t e =
            inline_table
                ? launch(stats_partial_kernel<true>, kKernelStatsPartial, n_tiles, kBlock, stream, a,
                         extra_lds)
                : launch(stats_partial_kernel<false>, kKernelStatsPartial, n_tiles, kBlock, stream,
                         a, extra_lds);
        if (e != hipSuccess) return e;
    }
    return inline_table ? launch(stats_final_kernel<true>, kKernelStatsFinal, (uint32_t)f.n_layers,
                                 kFinalBlock, stream, f)
                        : launch(stats_final_kernel<false>, kKernelStatsFinal,
                                 (uint32_t)f.n_layers, kFinalBlock, stream, f);
}

}  // namespace adt
