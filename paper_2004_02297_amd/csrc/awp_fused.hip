// One asynchronous pass of the whole path with device-resident AWP state
// (gfx950): statistics -> AWP rule -> Bitpack -> Bitunpack of arXiv 2004.02297
// (Section II / Algorithm 1, Section III / Algorithms 2 and 5) without a host
// round trip and with the weights read from HBM once.
//
// The byte count of a layer changes at most a handful of times in a whole
// training run (Algorithm 1 adds N bits after INTERVAL counted batches), so the
// pass speculates that this batch keeps the previous batch's byte counts:
//   1. fused kernel      : every wave tile of 1024 weights is loaded once; its
//                          sum of squares and largest magnitude go to a partial
//                          of its own, its top r bytes go to the packed stream
//                          and the truncated words (what Bitunpack would
//                          return) go to the output weights.
//   2. final + rule      : the partials of every layer are reduced in a fixed
//                          order (big layers by several sub-blocks), then
//                          Algorithm 1 runs per layer group: new bit count,
//                          interval counter, byte counts of the group's layers,
//                          and the flag `changed` if a byte count moved.
//   3. redo kernel       : a small grid that returns at once unless `changed`
//                          is set; then every block rebuilds the stream offsets
//                          (prefix sum of n_l * r_l) and the grid packs and
//                          truncates again with the new byte counts.
// The result is what statistics -> rule -> pack -> unpack would give in that
// order, whether or not the speculation held.
//
// While the host can prove that no byte count can move in a batch (no interval
// counter can reach INTERVAL: see begin_batch and plan_step), step 3 is not
// launched and step 2 does not get a launch of its own: its sub-blocks ride at
// the head of the NEXT batch's fused kernel, so that a batch is one launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_launch.h"
#include "adt_tables.h"
#include "adt_tile_ops.h"
#include "awp_partials.h"

namespace adt {

// Truncated words of a loaded wave tile -> output weights (what unpack, or
// unpack to a 16-bit format, returns).  dst: the tile's first output element.
constexpr int kOutNone = -1;
template <int R, int OUT>
__device__ __forceinline__ void store_truncated(const u32x4 (&v)[kChunksPerLane],
                                                void *__restrict__ dst, int len, int lane) {
    const uint32_t mask = R == 4 ? 0xFFFFFFFFu : (0xFFFFFFFFu << (8 * (4 - R)));
    u32x4 u[kChunksPerLane];
#pragma unroll
    for (int j = 0; j < kChunksPerLane; ++j) u[j] = v[j] & mask;
    store_unpacked_tile<OUT>(dst, len, lane, u);
}

// One wave tile: load once, then statistics (this lane's share of the tile's
// sum of squares in `sum`, largest magnitude folded into `mag`), truncated
// words and stream bytes.
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
    // all stores of the wave in one burst at its end (2 bytes: 217 us; truncated
    // words first and the stream after the LDS pass: 220 us)
    stream_out_wave_tile<R>(v, stream, len, lds, lane, stream_nt);
    if (OUT != kOutNone) store_truncated<R, OUT>(v, wout, len, lane);
}

// The layer a block tile belongs to, and where the tile starts in it.
struct BlockTileRef {
    int layer;
    int r;               // byte count of the layer
    int64_t elem;        // absolute index of the tile's first weight
    int64_t in_layer;    // index of that weight inside its layer
    int64_t layer_size;
};

__device__ __forceinline__ BlockTileRef find_block_tile(const FusedArgs &a, uint32_t tile) {
    // largest lo with tile_off[lo] <= tile: sixteen pivots at once, then a binary
    // search inside the range they leave (no step at all up to sixteen layers)
    int lo = pivot_range(a.tile_pivots, a.pivot_step, tile);
    int hi = lo + a.pivot_step < a.n_layers ? lo + a.pivot_step : a.n_layers;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (table_load(a.tile_off, mid) <= tile) lo = mid; else hi = mid;
    }
    BlockTileRef t;
    t.layer = lo;
    const int64_t e_begin = table_load(a.elem_off, lo);
    t.layer_size = table_load(a.elem_off, lo + 1) - e_begin;
    t.in_layer = (int64_t)(tile - table_load(a.tile_off, lo)) * kBlockTile;
    t.elem = e_begin + t.in_layer;
    t.r = table_byte(a.rbytes, lo);
    return t;
}

// Wave tile k (0..3) of a block tile.  layer_stream: where the layer's stream
// starts (from the table in global memory in the speculative pass, from the
// table rebuilt in LDS in the redo pass).
template <bool STATS, int OUT>
__device__ __forceinline__ void fused_block_wave_tile(const FusedArgs &a, const BlockTileRef &t,
                                                      int64_t layer_stream, bool stream_nt,
                                                      int k, int lane, uint32_t *lds,
                                                      double &sum, uint32_t &mag) {
    const int64_t first = t.in_layer + (int64_t)k * kWaveTile;
    const int64_t left = t.layer_size - first;
    const int len = __builtin_amdgcn_readfirstlane(
        left <= 0 ? 0 : (left < kWaveTile ? (int)left : kWaveTile));
    if (len == 0) return;
    const int64_t e = t.elem + (int64_t)k * kWaveTile;
    const uint32_t *src = a.weights + e;
    uint8_t *stream = a.packed + layer_stream + first * t.r;
    void *wout = OUT == kOutNone ? nullptr
                 : OUT == kOutFp32 ? (void *)((uint32_t *)a.weights_out + e)
                                   : (void *)((uint16_t *)a.weights_out + e);
    switch (t.r) {
        case 1: fused_wave_tile<1, STATS, OUT>(src, stream, wout, len, lds, lane, stream_nt, sum, mag); break;
        case 2: fused_wave_tile<2, STATS, OUT>(src, stream, wout, len, lds, lane, stream_nt, sum, mag); break;
        case 3: fused_wave_tile<3, STATS, OUT>(src, stream, wout, len, lds, lane, stream_nt, sum, mag); break;
        default: fused_wave_tile<4, STATS, OUT>(src, stream, wout, len, lds, lane, stream_nt, sum, mag); break;
    }
}

// Statistics of every layer, then Algorithm 1 for every group.  Phase 1: a
// sub-block reduces its chunk of one layer's partials (fixed order, see
// kFinalSlice) to a sub-partial.  Phase 2: the sub-block that finishes last
// among the sub-blocks of a group (a ticket counter per group, the one place in
// the library where a block reads what another block of the same launch wrote)
// adds up each of the group's layers from its sub-partials, again in an order
// fixed by the indices alone, writes the statistics and runs the rule for the
// group.  Which sub-block happens to be last has no influence on any result,
// and neither has the launch the sub-blocks ride in (a kernel of their own, or
// the head of the next batch's fused kernel).
struct FinalWork {          // what a sub-block's first wavefront knows before the reduction
    int g, layer, n_subs, l0, l1;
    uint32_t begin, end;
    int bits, counter, seen;    // lane 0 only
    double prev;                // lane 0 only
};

__device__ __forceinline__ FinalWork final_work(const FinalRuleArgs &a, uint32_t sub, int lane) {
    const uint32_t *sub_words = (const uint32_t *)a.subs + 4 * (size_t)sub;   // a FinalSub
    FinalWork w;
    w.g = (int)table_load(sub_words, 0);
    w.layer = (int)table_load(sub_words, 1);
    w.begin = table_load(sub_words, 2);
    w.end = table_load(sub_words, 3);
    w.n_subs = table_load(a.group_subs, w.g);
    w.l0 = table_load(a.group_off, w.g);
    w.l1 = table_load(a.group_off, w.g + 1);
    // what the rule will need, requested early so that it arrives behind the partials
    w.bits = w.counter = w.seen = 0;
    w.prev = 0.0;
    if (lane == 0) {
        w.bits = a.bits[w.g];
        w.counter = a.counter[w.g];
        w.prev = a.l2_prev[w.g];
        w.seen = *a.seen;
    }
    return w;
}

// Slice i of a chunk [begin, end): one wavefront, every lane returns the result.
__device__ __forceinline__ void reduce_slice(const FinalRuleArgs &a, const FinalWork &w, int i,
                                             int lane, double &sumsq, uint32_t &magnitude) {
    const uint32_t from = w.begin + (uint32_t)i * kFinalSlice;
    const uint32_t to = w.end - from > kFinalSlice ? from + kFinalSlice : w.end;
    sumsq = 0.0;
    magnitude = 0u;
    if (from < w.end)       // wave uniform
        wave_reduce_partials(a.partial_sumsq, a.partial_absmax, from, to, lane, sumsq, magnitude);
}

// Everything after the chunk's total (tot, tm: the same in all 64 lanes of the
// one wavefront that calls this).
__device__ __forceinline__ void final_rule_tail(const FinalRuleArgs &a, const FinalWork &w,
                                                uint32_t sub, int lane, double tot, uint32_t tm) {
    const int g = w.g;
    double group_sumsq = 0.0;
    if (w.n_subs == 1) {
        // one sub-block, hence at most one layer: no exchange with other blocks
        if (lane == 0 && w.layer >= 0) {
            double *o = a.stats + (int64_t)w.layer * 3;
            o[0] = tot;
            o[1] = sqrt(tot);
            o[2] = (double)__uint_as_float(tm);   // NaN bits stay NaN
            group_sumsq = tot;
        }
    } else {
        // The sub-partial is handed over through device-scope atomics, which act
        // where all XCDs see them: two exchanges, and only when both have returned
        // (the empty asm statement consumes their results) the ticket is drawn.  The
        // last sub-block reads the sub-partials with device-scope atomic loads.  No
        // cache is written back or invalidated on the way; a release / acquire fence
        // pair here stalls the whole memory system for some 80 ns, which the fused
        // kernel that carries these sub-blocks would pay for.
        int is_last = 0;
        if (lane == 0) {
            const unsigned long long was_s = atomicExch(
                (unsigned long long *)(a.sub_sumsq + sub), (unsigned long long)__double_as_longlong(tot));
            const uint32_t was_m = atomicExch(a.sub_absmax + sub, tm);
            asm volatile("" ::"v"((uint32_t)was_s), "v"((uint32_t)(was_s >> 32)), "v"(was_m) : "memory");
            const int ticket = atomicAdd(&a.group_ticket[g], 1);
            is_last = ticket == w.n_subs - 1;
        }
        if (__builtin_amdgcn_readfirstlane(is_last) == 0) return;   // lane 0's verdict
        // The group's norm is the l2-norm over all weights of its layers: the
        // layers' sums of squares added in index order.
        for (int l = w.l0; l < w.l1; ++l) {
            wave_reduce_partials<true>(a.sub_sumsq, a.sub_absmax, table_load(a.layer_sub_off, l),
                                       table_load(a.layer_sub_off, l + 1), lane, tot, tm);
            if (lane == 0) {
                double *o = a.stats + (int64_t)l * 3;
                o[0] = tot;
                o[1] = sqrt(tot);
                o[2] = (double)__uint_as_float(tm);
                group_sumsq += tot;
            }
        }
        if (lane == 0) a.group_ticket[g] = 0;                   // ready for the next pass
    }
    if (lane != 0) return;
    int bits = w.bits, counter = w.counter;
    const double now = sqrt(group_sumsq);
    if (w.seen != 0) {                      // the first batch only records its norm
        const double delta =
            w.prev == 0.0 ? (now == 0.0 ? 0.0 : __builtin_huge_val()) : (now - w.prev) / w.prev;
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
    bool moved = false;
    for (int l = w.l0; l < w.l1; ++l) {
        if (r != (int)a.rbytes[l]) {
            a.rbytes[l] = (uint8_t)r;
            moved = true;
        }
    }
    if (moved) *a.changed = 1;              // benign race: every writer stores 1
}

// A sub-block done by one wavefront (all 64 lanes active): the slices one after
// the other.
__device__ __forceinline__ void final_rule_wave(const FinalRuleArgs &a, uint32_t sub, int lane) {
    const FinalWork w = final_work(a, sub, lane);
    double tot = 0.0;
    uint32_t tm = 0u;
    for (int i = 0; i < a.n_slices; ++i) {
        double s;
        uint32_t m;
        reduce_slice(a, w, i, lane, s, m);
        tot += s;
        tm = m > tm ? m : tm;
    }
    final_rule_tail(a, w, sub, lane, tot, tm);
}

// A sub-block done by a block of up to sixteen wavefronts: one slice each, then
// the first wavefront adds the slice sums in index order and goes on alone.
__global__ __launch_bounds__(kFinalBlock) void final_rule_kernel(const FinalRuleArgs a) {
    static_assert(kFinalBlock == kFinalMaxSlices * kWave, "one wavefront per slice");
    __shared__ double slice_sum[kFinalMaxSlices];
    __shared__ uint32_t slice_mag[kFinalMaxSlices];
    const int lane = (int)(threadIdx.x & 63), wave = (int)(threadIdx.x >> 6);
    const FinalWork w = final_work(a, blockIdx.x, wave == 0 ? lane : 1);   // state: first lane only
    if (wave < a.n_slices) {
        double s;
        uint32_t m;
        reduce_slice(a, w, wave, lane, s, m);
        if (lane == 0) {
            slice_sum[wave] = s;
            slice_mag[wave] = m;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    double tot = 0.0;
    uint32_t tm = 0u;
    for (int i = 0; i < a.n_slices; ++i) {
        tot += slice_sum[i];
        tm = slice_mag[i] > tm ? slice_mag[i] : tm;
    }
    final_rule_tail(a, w, blockIdx.x, lane, tot, tm);
}

// The first wavefront, before anything of the batch is reduced: clears
// `changed`, hands the rule the "has a batch been seen" flag as it was before
// this batch, and publishes to the host how far the interval counters have got.
// A byte count can only move in a batch that takes some counter to INTERVAL
// (Algorithm 1), and a counter grows by at most one per batch, so the host can
// tell from an old status word that the next batches cannot change anything
// (see plan_step).  When the previous batch's rule is carried by this very
// launch, a counter may be read before or after that rule advances it: either
// value is at least what the batch before left, which is all the host assumes
// (and no counter is reset in a launch that carries a rule: the host has shown
// that none can reach INTERVAL).  All 64 lanes must be active.
__device__ __forceinline__ void begin_batch(const FusedArgs &a, int lane) {
    uint32_t top = 0u;
    for (int g = lane; g < a.n_status_groups; g += kWave) {
        const uint32_t c = (uint32_t)a.counter[g];
        top = c > top ? c : top;
    }
    top = wave_max(top);
    if (lane != 0) return;
    *a.changed = 0;                     // raised by the rule if need be
    *a.rule_seen = *a.steps_done;
    *a.steps_done = 1;
    const uint32_t begun = *a.batch_count;
    *a.batch_count = begun + 1u;
    if (a.host_status)
        __hip_atomic_store(a.host_status, ((unsigned long long)begun << 32) | top, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
}

// Speculative pass.  Wave tile number wt = 4 * (block tile) + k gets one
// wavefront, which writes one statistics partial, partial[wt]; no wavefront
// talks to another one.  The launch shape only decides how the wavefronts are
// grouped into blocks: four per block (block = block tile) or one per block
// (then a compute unit can be filled in steps of one wave, which is what the
// occupancy caps of the launchers need to work well).  Results do not depend
// on the shape.
template <int OUT, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void fused_kernel(const FusedArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[WAVES][kWaveLdsDw];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    uint32_t block = blockIdx.x;
    if (WAVES == 1 && a.n_pending_subs != 0u) {
        // the head of the grid carries the previous batch's final reduction and rule
        if (block < a.n_pending_subs) {
            final_rule_wave(a.pending, block, lane);
            return;
        }
        block -= a.n_pending_subs;
    }
    const uint32_t wt = WAVES == 1 ? block : block * (uint32_t)kWavesPerBlock + (uint32_t)wave;
    if (wt == 0) begin_batch(a, lane);        // wave uniform
    const BlockTileRef t = find_block_tile(a, wt / kWavesPerBlock);
    const bool nt = table_load(a.pack_off, a.n_layers) > a.stream_cache_limit;   // whole stream
    double sum = 0.0;
    uint32_t mag = 0u;
    fused_block_wave_tile<true, OUT>(a, t, table_load(a.pack_off, t.layer), nt,
                                     (int)(wt % kWavesPerBlock), lane, smem[wave], sum, mag);
    sum = wave_sum(sum);       // a wave tile beyond its layer's end contributes zeros
    mag = wave_max(mag);
    if (lane == 0) {
        a.partial_sumsq[wt] = sum;
        a.partial_absmax[wt] = mag;
    }
}

// Stream offsets of the current byte counts: exclusive prefix sum of n_l * r_l
// over the layers into out[0..n_layers] (global or LDS), by one block of
// `threads` threads (a multiple of 64, at most 1024).  Ends with a barrier.
__device__ __forceinline__ void block_prefix_pack_off(const int64_t *__restrict__ elem_off,
                                                      const uint8_t *__restrict__ rbytes,
                                                      int n_layers, int threads, int64_t *out) {
    __shared__ long long carry;
    __shared__ long long wave_total[kFinalWaves];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n_layers; base += threads) {
        const int l = base + tid;
        long long size = 0;
        if (l < n_layers) size = (long long)(elem_off[l + 1] - elem_off[l]) * (int)rbytes[l];
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
        if (l < n_layers) out[l] = before + incl - size;
        __syncthreads();
        if (tid == threads - 1) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) out[n_layers] = carry;
    __syncthreads();
}

// Plans with more layers than the redo kernel's LDS table holds: the stream
// offsets are rebuilt in global memory by this one-block kernel instead.
__global__ __launch_bounds__(kFinalBlock) void prefix_kernel(const FusedArgs a, int64_t *pack_off,
                                                             int64_t *packed_size) {
    if (*a.changed == 0) return;
    block_prefix_pack_off(a.elem_off, a.rbytes, a.n_layers, kFinalBlock, pack_off);
    if (threadIdx.x == 0) *packed_size = pack_off[a.n_layers];
}

// Redo pass: does nothing unless the rule changed a byte count.  LDS_TABLE:
// every block computes the new stream offsets into LDS for itself and block 0
// also stores them for the batches to come; otherwise they were rebuilt in
// global memory by prefix_kernel.
template <int OUT, bool LDS_TABLE>
__global__ __launch_bounds__(kBlock) void redo_kernel(const FusedArgs a, int64_t *pack_off_out,
                                                      int64_t *packed_size_out,
                                                      int32_t *steps_done) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[kWavesPerBlock][kWaveLdsDw];
    __shared__ int64_t lds_pack_off[LDS_TABLE ? kRedoLdsLayers + 1 : 1];
    if (blockIdx.x == 0 && threadIdx.x == 0) *steps_done = 1;   // a batch has been seen
    if (*a.changed == 0) return;
    const int64_t *pack_off = a.pack_off;
    if (LDS_TABLE) {
        block_prefix_pack_off(a.elem_off, a.rbytes, a.n_layers, kBlock, lds_pack_off);
        if (blockIdx.x == 0) {
            for (int l = (int)threadIdx.x; l <= a.n_layers; l += kBlock) pack_off_out[l] = lds_pack_off[l];
            if (threadIdx.x == 0) *packed_size_out = lds_pack_off[a.n_layers];
        }
        pack_off = lds_pack_off;
    }
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const bool nt = pack_off[a.n_layers] > a.stream_cache_limit;
    for (uint32_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        double sum = 0.0;
        uint32_t mag = 0u;
        const BlockTileRef t = find_block_tile(a, tile);
        fused_block_wave_tile<false, OUT>(a, t, pack_off[t.layer], nt, wave, lane, smem[wave], sum,
                                          mag);
        wave_lds_sync();     // the slice is reused by the next tile
    }
}

// Pack and truncate in one kernel from host-built tables (adt_pack_unpack): the
// weights are read once and both the stream and the words Bitunpack would
// return are written.  Blocks of WAVES wavefronts, one wave tile per wave.
template <bool INLINE, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void pack_unpack_kernel(const PackUnpackArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[WAVES][kWaveLdsDw];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const TileRef t = locate<INLINE, WAVES>(a.p, blockIdx.x, wave);
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

template <int WAVES>
static hipError_t launch_fused_w(const FusedArgs &a, int out_format, uint32_t extra_lds,
                                 hipStream_t stream) {
    void (*k)(FusedArgs) = out_format == kOutNone   ? fused_kernel<kOutNone, WAVES>
                           : out_format == kOutFp32 ? fused_kernel<kOutFp32, WAVES>
                           : out_format == kOutBf16 ? fused_kernel<kOutBf16, WAVES>
                                                    : fused_kernel<kOutFp16, WAVES>;
    const uint32_t carried = WAVES == 1 ? a.n_pending_subs : 0u;
    return launch(k, kKernelFused, a.n_tiles * (uint32_t)(kWavesPerBlock / WAVES) + carried,
                  WAVES * kWave, stream, a, extra_lds);
}

// out_format: kOutNone, kOutFp32, kOutBf16 or kOutFp16; waves: 1 or 4
hipError_t launch_fused(const FusedArgs &a, int out_format, int waves, uint32_t extra_lds,
                        hipStream_t stream) {
    return waves == 1 ? launch_fused_w<1>(a, out_format, extra_lds, stream)
                      : launch_fused_w<4>(a, out_format, extra_lds, stream);
}

hipError_t launch_final_rule(const FinalRuleArgs &a, hipStream_t stream) {
    return launch(final_rule_kernel, kKernelFinalRule, (uint32_t)a.n_subs, kFinalBlock, stream, a);
}

template <typename... A>
static hipError_t launch_plain(void (*kernel)(A...), int kernel_id, uint32_t grid, int block,
                               hipStream_t stream, A... args) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (timing_events(kernel_id, stream, &e0, &e1))
        hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, stream, e0, e1, 0, args...);
    else
        kernel<<<dim3(grid), dim3(block), 0, stream>>>(args...);
    return hipGetLastError();
}

hipError_t launch_redo(const FusedArgs &a, int out_format, int64_t *pack_off, int64_t *packed_size,
                       int32_t *steps_done, hipStream_t stream) {
    const bool lds_table = a.n_layers <= kRedoLdsLayers;
    if (!lds_table) {
        hipError_t e = launch_plain(prefix_kernel, kKernelPrefix, 1u, kFinalBlock, stream, a, pack_off,
                                    packed_size);
        if (e != hipSuccess) return e;
    }
    uint32_t grid = a.n_tiles < (uint32_t)kRedoBlocks ? a.n_tiles : (uint32_t)kRedoBlocks;
    if (grid == 0) grid = 1;
    void (*k)(FusedArgs, int64_t *, int64_t *, int32_t *);
    if (lds_table)
        k = out_format == kOutNone   ? redo_kernel<kOutNone, true>
            : out_format == kOutFp32 ? redo_kernel<kOutFp32, true>
            : out_format == kOutBf16 ? redo_kernel<kOutBf16, true>
                                     : redo_kernel<kOutFp16, true>;
    else
        k = out_format == kOutNone   ? redo_kernel<kOutNone, false>
            : out_format == kOutFp32 ? redo_kernel<kOutFp32, false>
            : out_format == kOutBf16 ? redo_kernel<kOutBf16, false>
                                     : redo_kernel<kOutFp16, false>;
    return launch_plain(k, kKernelRedo, grid, kBlock, stream, a, pack_off, packed_size, steps_done);
}

// waves: 1 or 4 (the tile table must have been built for waves * 1024 weights per block)
hipError_t launch_pack_unpack(const PackUnpackArgs &a, uint32_t n_tiles, bool inline_table,
                              int waves, uint32_t extra_lds, hipStream_t stream) {
    void (*k)(PackUnpackArgs);
    if (waves == 1) k = inline_table ? pack_unpack_kernel<true, 1> : pack_unpack_kernel<false, 1>;
    else k = inline_table ? pack_unpack_kernel<true, 4> : pack_unpack_kernel<false, 4>;
    return launch(k, kKernelPackUnpack, n_tiles, waves * kWave, stream, a, extra_lds);
}

}  // namespace adt
