// Per-layer tables shared by the host launcher and the gfx950 kernels.
//
// One launch covers all layers: the grid is the concatenation of every
// layer's tiles, and a block finds its layer by a binary search over
// tile_off.  Tables of up to ADT_INLINE_LAYERS layers travel inside the
// kernel-argument buffer (no copy, no lifetime to manage); larger ones are
// staged through a ring of device buffers.
#pragma once

#include <stdint.h>

namespace adt {

constexpr int kWave = 64;               // CDNA wavefront
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
#ifndef ADT_CHUNKS_PER_LANE
#define ADT_CHUNKS_PER_LANE 4
#endif
constexpr int kChunksPerLane = ADT_CHUNKS_PER_LANE;   // 128-bit loads in flight per lane
constexpr int kWaveTile = kWave * kChunksPerLane * 4;    // 1024 weights per wave
constexpr int kBlockTile = kWaveTile * kWavesPerBlock;   // 4096 weights per block
// Unpack always runs one wavefront per block; pack, pack + unpack and the
// fused kernel of the plan can run one or four (see "launch shapes" below).
constexpr int kUnpackWaves = 1;
constexpr int kUnpackBlockTile = kWaveTile * kUnpackWaves;

// Statistics kernel: 8 128-bit loads per lane, 8192 weights per block.
constexpr int kStatsLoadsPerLane = 8;
constexpr int kStatsTile = kBlock * kStatsLoadsPerLane * 4;

// Launch shapes.  On MI355X a streaming kernel sustains the most bandwidth with
// far fewer waves in flight than a compute unit could hold (32): measured on
// 138 M weights with rotating output buffers (so that the last-level cache
// cannot absorb rewrites), the kernels that write more than they read are
// fastest with 7 to 13 waves per compute unit and lose 5 to 10 % at 32.  Two
// things make such a low occupancy work: blocks of ONE wavefront, so that a
// compute unit is refilled the moment any wave retires (a four-wave block holds
// the slots of its finished waves until the last one drains), and a wave that
// reaches its first streaming load without any vector-memory round trip (all
// table look-ups are scalar loads, see table_load).  The launchers request
// dynamic LDS that no kernel touches; a compute unit has 160 KB, a one-wave
// block of the pack / unpack kernels owns 4160 B of its own:
//   extra 4 KB -> 19 waves, 6 KB -> 15, 8 KB -> 13, 10 KB -> 11, 12 KB -> 9,
//   14 KB -> 8, 16 KB -> 7.
// Microseconds per launch, 138 M weights, all layers at 1 / 2 / 3 / 4 bytes
// (one-wave blocks; streaming stores, see store_streaming16):
//   fused (plan),  4-wave blocks, no cap   223 / 250 / 283 / 298  (before the streaming stores)
//   FP32 truncated 8 KB                    196 / 219 / 249 / 269
//   weights        12 KB                   191 / 213 / 243 / 265
//                  14 KB                   200 / 218 / 239 / 261
//                  16 KB                   222 / 237 / 252 / 268
//   fused, 16-bit  6 KB                    148 / 173 / 200 / 219
//   truncated      8 KB                    148 / 171 / 201 / 220
//   weights        10 KB                   152 / 173 / 196 / 217
//                  12 KB                   157 / 178 / 197 / 215
//   pack + unpack  8 KB                    195 / 217 / 248 / 268
//                  12 KB                   190 / 215 / 243 / 266
//                  14 KB                   187 / 210 / 239 / 261
//                  16 KB                   193 / 212 / 236 / 257
//                  20 KB                   204 / 221 / 250 / 255
//   pack           4 KB, ordinary stores   105 / 120 /  -  /  -   (4-wave blocks: 112 / 129)
//                  4 KB, streaming stores  111 / 127 / 149 / 171
//                  10 KB, streaming stores 113 / 132 / 148 / 166
//   unpack         2 KB                    112 / 134 / 159 / 175  (no cap: 129 / 145 / 166 / 180)
//                  6 KB                    114 / 129 / 154 / 169
//                  12 KB                   136 / 132 / 151 / 166
//   right behind   6 KB                    117 / 114 / 154 / 168
//   pack           12 KB                   140 / 117 / 151 / 166
// The cap is chosen from the bytes written per weight (how write-heavy the
// launch is).
struct LaunchShape {
    int waves;            // wavefronts per block: 1 or 4
    uint32_t extra_lds;   // bytes of dynamic LDS nothing touches
};
// written_per_weight: stream bytes plus the bytes of a truncated weight (4, 2 or 0)
inline LaunchShape fused_shape(double written_per_weight, int out_bytes) {
    if (out_bytes == 2)
        return LaunchShape{1, written_per_weight <= 4.5   ? 8192u
                              : written_per_weight <= 5.5 ? 10240u
                                                          : 12288u};
    if (out_bytes == 4) return LaunchShape{1, written_per_weight <= 6.5 ? 12288u : 14336u};
    // statistics and stream only (us at 1 / 2 / 3 / 4 bytes): 4 KB 108 / 126 / 150 / 172,
    // 8 KB 113 / 129 / 149 / 169, 10 KB 122 / 137 / 152 / 168; no cap 118 / 131 / 155 / 177
    return LaunchShape{1, written_per_weight <= 2.6 ? 4096u : written_per_weight <= 3.5 ? 8192u : 10240u};
}
inline LaunchShape pack_unpack_shape(double bytes_per_weight) {
    return LaunchShape{1, bytes_per_weight <= 2.6 ? 14336u : 16384u};
}
// streaming: the stream is larger than the size up to which pack keeps it in the cache
inline LaunchShape pack_shape(double, bool streaming) {
    return LaunchShape{1, streaming ? 10240u : 4096u};
}
// unpack to 16 bits reads about as much as it writes and wants more waves (2 KB:
// 68 / 85 / 110 / 127 us; 6 KB: 83 / 97 / 117 / 133 us)
inline LaunchShape unpack_shape(double bytes_per_weight, bool out16) {
    return LaunchShape{kUnpackWaves, out16 ? 2048u : bytes_per_weight <= 2.6 ? 6144u : 12288u};
}
// Statistics: 4-wave blocks of 8192 weights, 16 waves per compute unit (77 us for 138 M weights,
// 80 us uncapped or with any other cap; one- and two-wave blocks of 1024 - 4096 weights: 78 - 83 us
// and a longer final kernel).  A grid of a few blocks per compute unit runs uncapped: with the cap
// 3113 blocks (25 M weights) make just over three rounds of 1024 resident blocks, 15.4 us against 14.1.
inline LaunchShape stats_shape(uint32_t n_tiles) {
    return LaunchShape{4, n_tiles <= 4096u ? 0u : 36864u};
}

constexpr int kInlineLayers = 128;

#if defined(__HIPCC__)
// Wave-uniform read of a table entry that nothing writes while the kernel runs.
// The read goes through the constant address space: that tells the compiler the
// data is invariant, so it issues a scalar load.  Through an ordinary global
// pointer it would issue a vector memory load, and a block's binary search over
// the table would become a chain of round trips through the (saturated) vector
// memory pipeline before the wave can issue its first streaming load.
template <typename T>
__device__ __forceinline__ T table_load(const T *table, int64_t idx) {
    typedef const T __attribute__((address_space(4))) *ConstantPtr;
    return ((ConstantPtr)table)[idx];
}

// Entry idx of a byte table through a scalar dword load (there is no scalar
// byte load).  The table must be 4-byte aligned and readable up to the next
// multiple of four entries; idx must be wave uniform.
__device__ __forceinline__ int table_byte(const uint8_t *table, int idx) {
    const uint32_t word = table_load((const uint32_t *)table, idx >> 2);
    return (int)((word >> (8 * (idx & 3))) & 0xFFu);
}

// Sixteen table entries with one scalar load (the table must be 64-byte
// aligned).  A wave's life at the occupancy these kernels run at is a few
// microseconds, and every dependent look-up before its first streaming load is
// a round trip of that life: the first level of the tile search therefore reads
// sixteen pivots at once and compares them in scalar registers.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ u32x16 table_load16(const uint32_t *table) {
    typedef const u32x16 __attribute__((address_space(4))) *ConstantPtr;
    return *(ConstantPtr)table;
}
// pivots[i] = tile_off[min(i * step, n_layers)], i = 0..15 (see tile_pivots).
// Returns the first layer of the range of `step` layers that holds `tile`.
__device__ __forceinline__ int pivot_range(const uint32_t *pivots, int step, uint32_t tile) {
    const u32x16 p = table_load16(pivots);
    int c = 0;
#pragma unroll
    for (int i = 1; i < 16; ++i) c += p[i] <= tile ? 1 : 0;     // the pivots do not decrease
    return c * step;
}
#endif

// First level of the tile search: sixteen pivots out of tile_off (n_layers + 1
// entries, non-decreasing), `step` layers apart; returns step.
constexpr int kTilePivots = 16;
inline int tile_pivots(const uint32_t *tile_off, int n_layers, uint32_t *pivots) {
    const int step = n_layers <= kTilePivots ? 1 : (n_layers + kTilePivots - 1) / kTilePivots;
    for (int i = 0; i < kTilePivots; ++i) {
        const int64_t l = (int64_t)i * step;
        pivots[i] = tile_off[l < n_layers ? l : n_layers];
    }
    return step;
}

// Layer l covers weights [elem_off[l], elem_off[l+1]), packed bytes
// [pack_off[l], pack_off[l+1]) and tiles [tile_off[l], tile_off[l+1]).
struct InlineTable {
    int64_t elem_off[kInlineLayers + 1];
    int64_t pack_off[kInlineLayers + 1];
    uint32_t tile_off[kInlineLayers + 1];
    uint8_t rbytes[kInlineLayers];
};

struct DeviceTable {
    const int64_t *elem_off;
    const int64_t *pack_off;
    const uint32_t *tile_off;
    const uint8_t *rbytes;
};

struct PackArgs {
    const uint32_t *weights;   // FP32 words, read by pack / written by unpack
    uint8_t *packed;           // dense stream
    int64_t packed_size;       // bytes in the whole stream
    int64_t stream_cache_limit;   // streams larger than this are written nontemporal
    int n_layers;
    DeviceTable dev;           // used when n_layers > kInlineLayers
    InlineTable inl;
};

// adt_pack_unpack: pack plus the truncated FP32 copy in one kernel.
struct PackUnpackArgs {
    PackArgs p;
    uint32_t *weights_out;
};

struct StatsInlineTable {
    int64_t elem_off[kInlineLayers + 1];
    uint32_t tile_off[kInlineLayers + 1];
};

struct StatsArgs {
    const uint32_t *weights;
    double *partial_sumsq;     // one per tile
    uint32_t *partial_absmax;  // one per tile, magnitude bits
    int n_layers;
    const int64_t *dev_elem_off;
    const uint32_t *dev_tile_off;
    StatsInlineTable inl;
};

struct StatsFinalArgs {
    const double *partial_sumsq;
    const uint32_t *partial_absmax;
    double *stats_out;         // n_layers x 3
    int n_layers;
    const uint32_t *dev_tile_off;
    uint32_t inl_tile_off[kInlineLayers + 1];
};

// Ablation kernels (adt_ablation.hip): inline tables only.
constexpr int kNaiveTile = kBlock;        // one weight per thread
constexpr int kVecTile = kBlock * 4;      // four weights per thread
struct AblationArgs {
    const uint32_t *weights;
    uint8_t *packed;
    int n_layers;
    int64_t elem_off[kInlineLayers + 1];
    int64_t pack_off[kInlineLayers + 1];
    uint32_t tile_off[kInlineLayers + 1];   // tiles of kNaiveTile / kVecTile weights
    uint8_t rbytes[kInlineLayers];
};

// Final reduction of the statistics + Algorithm 1.  The partials of a layer
// are cut into chunks, the work of one "sub-block"; a chunk is n_slices slices
// of kFinalSlice partials.  A slice is summed by one
// wavefront (eight partials per lane, then across the lanes), the slices of a
// chunk are added in index order.  That order does not depend on who does the
// work: the sixteen wavefronts of a block, one slice each (the kernel of its
// own), or one wavefront walking the slices (a sub-block carried at the head of
// the next batch's fused kernel).  Every layer has at least one sub-block (an
// empty layer: an empty chunk) and every group at least one (a group without
// layers: one that reduces nothing), so that each group's rule runs.
// A plan picks the slices per chunk (1 .. kFinalMaxSlices) from its size, so
// that a carried sub-block, whose one wavefront needs a memory round trip per
// slice, stays short next to the fused kernel that carries it.
constexpr uint32_t kFinalSlice = 512;
constexpr int kFinalMaxSlices = 16;
inline int final_slices_for(uint64_t n_partials) {      // aims at about 32 sub-blocks of big layers
    const uint64_t want = (n_partials + 32 * kFinalSlice - 1) / (32 * kFinalSlice);
    return want < 1 ? 1 : want > (uint64_t)kFinalMaxSlices ? kFinalMaxSlices : (int)want;
}
struct FinalSub {           // work of one sub-block
    int32_t group;
    int32_t layer;          // -1: the group has no layer
    uint32_t begin, end;    // partials [begin, end) of that layer
};
struct FinalRuleArgs {
    const double *partial_sumsq;    // the partials of the batch to reduce
    const uint32_t *partial_absmax;
    const FinalSub *subs;           // one per sub-block
    const uint32_t *layer_sub_off;  // n_layers + 1: sub-blocks of layer l are [off[l], off[l+1])
    const int32_t *group_subs;      // per group: number of its sub-blocks
    int32_t *group_ticket;          // per group: sub-blocks finished in this pass (0 between passes)
    double *sub_sumsq;              // one per sub-block
    uint32_t *sub_absmax;
    double *stats;              // n_layers x 3
    const int32_t *group_off;   // n_groups + 1 layer indices
    int n_subs;
    int n_slices;               // slices per chunk
    double *l2_prev;            // per group
    int32_t *bits;              // per group
    int32_t *counter;           // per group
    uint8_t *rbytes;            // per layer
    int32_t *changed;
    const int32_t *seen;        // 0 for the first batch: that batch only records norms
    double T;
    int interval;
    int n_bits;
};

// Device-resident tables of a plan (see awp_fused.hip): everything is a
// device pointer; tile_off counts block tiles of kBlockTile weights.
struct FusedArgs {
    const uint32_t *weights;
    uint8_t *packed;
    void *weights_out;          // FP32 words or 16-bit elements; null: no truncated copy
    const int64_t *elem_off;
    const int64_t *pack_off;
    const uint32_t *tile_off;
    const uint32_t *tile_pivots;    // kTilePivots entries, 64-byte aligned (see tile_pivots)
    int pivot_step;
    const uint8_t *rbytes;
    double *partial_sumsq;      // one per wave tile: 4 * n_tiles entries (this batch's set)
    uint32_t *partial_absmax;
    int32_t *changed;           // cleared by the fused kernel, raised by the rule, read by redo
    // Bookkeeping of a batch, done by the fused kernel's first wavefront before
    // anything of the batch is reduced (see begin_batch in awp_fused.hip):
    int32_t *steps_done;        // non-zero once a batch has been processed
    int32_t *rule_seen;         // steps_done as it was before this batch: what this batch's rule reads
    uint32_t *batch_count;      // batches begun since the plan was created or its state set
    const int32_t *counter;     // per group: interval counters (the previous batches' rule wrote them)
    int n_status_groups;        // number of groups if the status word is kept, else 0
    unsigned long long *host_status;   // pinned host word (batches << 32 | largest counter); may be null
    int64_t stream_cache_limit;   // streams larger than this are written nontemporal
    int n_layers;
    uint32_t n_tiles;
    // The previous batch's final reduction and rule, carried along by the first
    // n_pending_subs one-wave blocks of this launch (0: nothing is carried).
    uint32_t n_pending_subs;
    FinalRuleArgs pending;
};

// Redo pass: layers whose stream-offset table fits the kernel's LDS, and its grid.
constexpr int kRedoLdsLayers = 1024;
constexpr int kRedoBlocks = 1024;
// Plans with more groups than this do not publish the largest interval counter
// (one wavefront scans the counters at the start of every batch) and launch the
// redo pass with every batch.
constexpr int kStatusMaxGroups = 4096;

}  // namespace adt
