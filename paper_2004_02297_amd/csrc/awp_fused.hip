// One asynchronous pass of the whole path with device-resident AWP state
// (gfx950): statistics -> AWP rule -> Bitpack -> Bitunpack of arXiv 2004.02297
// (Section II / Algorithm 1, Section III / Algorithms 2 and 5) without a host
// round trip and with the weights read from HBM once.
//
// The byte count of a layer changes at most a handful of times in a whole
// training run (Algorithm 1 adds N bits after INTERVAL counted batches), so the
// pass speculates that this batch keeps the previous batch's byte counts:
//   1. fused kernel   : every wave tile of 1024 weights is loaded once; its
//                       sum of squares and largest magnitude go to a per-block
//                       partial, its top r bytes go to the packed stream and the
//                       truncated words (what Bitunpack would return) go to the
//                       output weights.
//   2. final kernel   : per-layer reduction of the partials (fixed order).
//   3. rule kernel    : one block runs Algorithm 1 on the fresh norms, rewrites
//                       the byte counts and the stream offsets (prefix sum) and
//                       raises `changed` if any byte count moved.
//   4. redo kernel    : a small persistent grid that returns at once unless
//                       `changed` is set; then it packs and truncates again with
//                       the new table.
// The result is what statistics -> rule -> pack -> unpack would give in that
// order, whether or not the speculation held.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_launch.h"
#include "adt_tables.h"
#include "adt_tile_ops.h"

namespace adt {

__device__ __forceinline__ double fused_wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ uint32_t fused_wave_max(uint32_t v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

__device__ __forceinline__ void square_add(uint32_t bits, double &acc, uint32_t &mag) {
    const double w = (double)__uint_as_float(bits);
    acc = fma(w, w, acc);               // the square of a binary32 is exact in binary64
    const uint32_t m = bits & 0x7FFFFFFFu;
    mag = m > mag ? m : mag;            // NaN patterns order above infinity
}

// Truncated words of a loaded wave tile -> output weights (what unpack, or
// unpack to a 16-bit format, returns).  dst: the tile's first output element.
constexpr int kOutNone = -1;
template <int R, int OUT>
__device__ __forceinline__ void store_truncated(const u32x4 (&v)[kChunksPerLane],
                                                void *__restrict__ dst, int len, int lane) {
    const uint32_t mask = R == 4 ? 0xFFFFFFFFu : (0xFFFFFFFFu << (8 * (4 - R)));
    const bool dst_dw = ((uintptr_t)dst & 3u) == 0;       // wave uniform
#pragma unroll
    for (int j = 0; j < kChunksPerLane; ++j) {
        const int e0 = 4 * (j * kWave + lane);
        if (e0 < len) store_unpacked<OUT>(dst, e0, len, v[j] & mask, dst_dw);
    }
}

template <int R, bool STATS, int OUT>
__device__ __forceinline__ void fused_wave_tile(const uint32_t *__restrict__ src,
                                                uint8_t *__restrict__ stream,
                                                void *__restrict__ wout, int len,
                                                uint32_t *lds, int lane, bool stream_nt,
                                                double &sum, uint32_t &mag) {
    u32x4 v[kChunksPerLane];
    load_wave_tile(src, len, lane, v);
    if (STATS) {
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll
        for (int j = 0; j < kChunksPerLane; ++j) {   // words past len are zero
            square_add(v[j].x, a0, mag);
            square_add(v[j].y, a1, mag);
            square_add(v[j].z, a2, mag);
            square_add(v[j].w, a3, mag);
        }
        sum = (a0 + a1) + (a2 + a3);
    }
    if (OUT != kOutNone) store_truncated<R, OUT>(v, wout, len, lane);
    stream_out_wave_tile<R>(v, stream, len, lds, lane, stream_nt);
}

template <bool STATS, int OUT>
__device__ __forceinline__ void fused_block_tile(const FusedArgs &a, uint32_t tile, int wave,
                                                 int lane, uint32_t *lds, double &sum,
                                                 uint32_t &mag) {
    int lo = 0, hi = a.n_layers;            // largest lo with tile_off[lo] <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_off[mid] <= tile) lo = mid; else hi = mid;
    }
    const int64_t e_begin = a.elem_off[lo];
    const int64_t first = (int64_t)(tile - a.tile_off[lo]) * kBlockTile + (int64_t)wave * kWaveTile;
    const int64_t left = (a.elem_off[lo + 1] - e_begin) - first;
    const int len = __builtin_amdgcn_readfirstlane(
        left <= 0 ? 0 : (left < kWaveTile ? (int)left : kWaveTile));
    if (len == 0) return;
    const int r = __builtin_amdgcn_readfirstlane((int)a.rbytes[lo]);
    const uint32_t *src = a.weights + e_begin + first;
    uint8_t *stream = a.packed + a.pack_off[lo] + first * r;
    void *wout = OUT == kOutNone ? nullptr
                 : OUT == kOutFp32 ? (void *)((uint32_t *)a.weights_out + e_begin + first)
                                   : (void *)((uint16_t *)a.weights_out + e_begin + first);
    const bool nt = a.pack_off[a.n_layers] > a.stream_cache_limit;   // whole stream's size
    switch (r) {
        case 1: fused_wave_tile<1, STATS, OUT>(src, stream, wout, len, lds, lane, nt, sum, mag); break;
        case 2: fused_wave_tile<2, STATS, OUT>(src, stream, wout, len, lds, lane, nt, sum, mag); break;
        case 3: fused_wave_tile<3, STATS, OUT>(src, stream, wout, len, lds, lane, nt, sum, mag); break;
        default: fused_wave_tile<4, STATS, OUT>(src, stream, wout, len, lds, lane, nt, sum, mag); break;
    }
}

// Speculative pass: one block tile (4096 weights) per block, statistics on.
template <int OUT>
__global__ __launch_bounds__(kBlock) void fused_kernel(const FusedArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[kWavesPerBlock][kWaveLdsDw];
    __shared__ double wsum[kWavesPerBlock];
    __shared__ uint32_t wmag[kWavesPerBlock];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    double sum = 0.0;
    uint32_t mag = 0u;
    fused_block_tile<true, OUT>(a, blockIdx.x, wave, lane, smem[wave], sum, mag);
    sum = fused_wave_sum(sum);
    mag = fused_wave_max(mag);
    if (lane == 0) {
        wsum[wave] = sum;
        wmag[wave] = mag;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a.partial_sumsq[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
        uint32_t m = wmag[0];
#pragma unroll
        for (int i = 1; i < kWavesPerBlock; ++i) m = wmag[i] > m ? wmag[i] : m;
        a.partial_absmax[blockIdx.x] = m;
    }
}

// Redo pass: persistent grid; does nothing unless the rule changed a byte count.
template <int OUT>
__global__ __launch_bounds__(kBlock) void redo_kernel(const FusedArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[kWavesPerBlock][kWaveLdsDw];
    if (*a.changed == 0) return;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    for (uint32_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        double sum = 0.0;
        uint32_t mag = 0u;
        fused_block_tile<false, OUT>(a, tile, wave, lane, smem[wave], sum, mag);
        wave_lds_sync();     // the slice is reused by the next tile
    }
}

// Pack and truncate in one kernel from host-built tables (adt_pack_unpack): the
// weights are read once and both the stream and the words Bitunpack would
// return are written.
template <bool INLINE>
__global__ __launch_bounds__(kBlock) void pack_unpack_kernel(const PackUnpackArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[kWavesPerBlock][kWaveLdsDw];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const TileRef t = locate<INLINE>(a.p, blockIdx.x, wave);
    if (t.len == 0) return;
    const uint32_t *src = a.p.weights + t.elem;
    uint8_t *stream = a.p.packed + t.byte;
    uint32_t *wout = a.weights_out + t.elem;
    uint32_t *lds = smem[wave];
    double sum = 0.0;
    uint32_t mag = 0u;
    const bool nt = a.p.packed_size > a.p.stream_cache_limit;
    switch (t.r) {
        case 1: fused_wave_tile<1, false, kOutFp32>(src, stream, wout, t.len, lds, lane, nt, sum, mag); break;
        case 2: fused_wave_tile<2, false, kOutFp32>(src, stream, wout, t.len, lds, lane, nt, sum, mag); break;
        case 3: fused_wave_tile<3, false, kOutFp32>(src, stream, wout, t.len, lds, lane, nt, sum, mag); break;
        default: fused_wave_tile<4, false, kOutFp32>(src, stream, wout, t.len, lds, lane, nt, sum, mag); break;
    }
}

// Algorithm 1 for all layers, then the stream offsets of the new byte counts.
constexpr int kRuleBlock = 1024;
constexpr int kRuleWaves = kRuleBlock / kWave;

__global__ __launch_bounds__(kRuleBlock) void rule_kernel(const RuleArgs a) {
    __shared__ int any_changed;
    __shared__ long long carry;
    __shared__ long long wave_total[kRuleWaves];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool is_first = *a.steps_done == 0;   // read by all before thread 0 bumps it at the end
    if (tid == 0) {
        any_changed = 0;
        carry = 0;
    }
    __syncthreads();
    // Phase 1: one thread per group.  The group's norm is the l2-norm over all
    // weights of its layers (sum of the layers' sums of squares, index order).
    for (int g = tid; g < a.n_groups; g += kRuleBlock) {
        const int l0 = a.group_off[g], l1 = a.group_off[g + 1];
        double sumsq = 0.0;
        for (int l = l0; l < l1; ++l) sumsq += a.stats[3 * l];
        const double now = sqrt(sumsq);
        int bits = a.bits[g];
        if (!is_first) {
            const double prev = a.l2_prev[g];
            const double delta =
                prev == 0.0 ? (now == 0.0 ? 0.0 : __builtin_huge_val()) : (now - prev) / prev;
            int counter = a.counter[g];
            if (delta < a.T) ++counter;
            if (counter == a.interval) {
                bits += a.n_bits;
                if (bits > 32) bits = 32;
                counter = 0;
            }
            a.counter[g] = counter;
            a.bits[g] = bits;
        }
        a.l2_prev[g] = now;
        const int r = (bits + 7) >> 3;
        for (int l = l0; l < l1; ++l) {
            if (r != (int)a.rbytes[l]) {
                a.rbytes[l] = (uint8_t)r;
                any_changed = 1;      // benign race: every writer stores 1
            }
        }
    }
    __syncthreads();
    // Phase 2: stream offsets = exclusive prefix sum of n_l * r_l over the layers.
    for (int base = 0; base < a.n_layers; base += kRuleBlock) {
        const int l = base + tid;
        long long size = 0;
        if (l < a.n_layers)
            size = (long long)(a.elem_off[l + 1] - a.elem_off[l]) * (int)a.rbytes[l];
        // exclusive prefix sum of `size` over the block, on top of `carry`
        long long incl = size;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const long long o = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += o;
        }
        if (lane == kWave - 1) wave_total[wave] = incl;
        __syncthreads();
        long long before = carry;
        for (int w = 0; w < wave; ++w) before += wave_total[w];
        if (l < a.n_layers) a.pack_off[l] = before + incl - size;
        __syncthreads();
        if (tid == kRuleBlock - 1) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) {
        a.pack_off[a.n_layers] = carry;
        *a.packed_size = carry;
        *a.changed = any_changed;
        *a.steps_done = 1;
    }
}

// out_format: kOutNone, kOutFp32, kOutBf16 or kOutFp16
hipError_t launch_fused(const FusedArgs &a, int out_format, hipStream_t stream) {
    void (*k)(FusedArgs) = out_format == kOutNone   ? fused_kernel<kOutNone>
                           : out_format == kOutFp32 ? fused_kernel<kOutFp32>
                           : out_format == kOutBf16 ? fused_kernel<kOutBf16>
                                                    : fused_kernel<kOutFp16>;
    return launch(k, kKernelFused, a.n_tiles, kBlock, stream, a);
}

hipError_t launch_redo(const FusedArgs &a, int out_format, hipStream_t stream) {
    const uint32_t grid = a.n_tiles < 1024u ? a.n_tiles : 1024u;
    void (*k)(FusedArgs) = out_format == kOutNone   ? redo_kernel<kOutNone>
                           : out_format == kOutFp32 ? redo_kernel<kOutFp32>
                           : out_format == kOutBf16 ? redo_kernel<kOutBf16>
                                                    : redo_kernel<kOutFp16>;
    return launch(k, kKernelRedo, grid, kBlock, stream, a);
}

hipError_t launch_pack_unpack(const PackUnpackArgs &a, uint32_t n_tiles, bool inline_table,
                              hipStream_t stream) {
    return inline_table
               ? launch(pack_unpack_kernel<true>, kKernelPackUnpack, n_tiles, kBlock, stream, a)
               : launch(pack_unpack_kernel<false>, kKernelPackUnpack, n_tiles, kBlock, stream, a);
}

hipError_t launch_rule(const RuleArgs &a, hipStream_t stream) {
    return launch(rule_kernel, kKernelRule, 1u, kRuleBlock, stream, a);
}

}  // namespace adt
