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
// Unpack runs one wavefront per block: its waves finish at uneven times (the
// stores dominate), and single-wave blocks let a new tile start the moment any
// wave slot frees up instead of when a whole four-wave block has drained
// (138 M weights at 2 bytes: 141 us instead of 151 us).
constexpr int kUnpackWaves = 1;
constexpr int kUnpackBlockTile = kWaveTile * kUnpackWaves;

// Statistics kernel: 8 128-bit loads per lane, 8192 weights per block.
constexpr int kStatsLoadsPerLane = 8;
constexpr int kStatsTile = kBlock * kStatsLoadsPerLane * 4;

// Waves in flight.  On MI355X a streaming kernel does not always sustain the
// most bandwidth with the 32 waves per compute unit the hardware could hold: a
// copy-like probe runs at 6.1 TB/s with 32 waves and 6.5 TB/s with 16, one read
// per two writes at 5.8 vs 6.6 TB/s, a pure read at 6.9 vs 7.2 TB/s.  Unpack
// (138 M weights, after pack, at 1 / 2 / 3 / 4 bytes: 119 / 117 / 156 / 173 us
// with 19 waves, 124 / 122 / 163 / 176 us uncapped; 15 waves are as good from
// 2 bytes up but cost 11 % at 1 byte) and the statistics kernel (76.9 vs
// 79.0 us with 16 waves) gain; pack and the fused kernel do not, and stay
// uncapped.  The launchers request this much dynamic LDS that no kernel
// touches, so that a compute unit (160 KB of LDS) holds fewer blocks:
constexpr uint32_t kUnpackExtraLds = 4096;    // 4.1 + 4 KB per 1-wave block -> 19 blocks
constexpr uint32_t kStatsExtraLds = 36864;    // 4-wave blocks               -> 4 blocks

constexpr int kInlineLayers = 128;

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

// Device-resident tables of a plan (see awp_fused.hip): everything is a
// device pointer; tile_off counts block tiles of kBlockTile weights.
struct FusedArgs {
    const uint32_t *weights;
    uint8_t *packed;
    void *weights_out;          // FP32 words or 16-bit elements; null: no truncated copy
    const int64_t *elem_off;
    const int64_t *pack_off;
    const uint32_t *tile_off;
    const uint8_t *rbytes;
    double *partial_sumsq;      // one per block tile
    uint32_t *partial_absmax;
    const int32_t *changed;
    int64_t stream_cache_limit;   // streams larger than this are written nontemporal
    int n_layers;
    uint32_t n_tiles;
};

struct RuleArgs {
    const double *stats;        // n_layers x 3, written by the final kernel
    const int32_t *group_off;   // n_groups + 1 layer indices
    int n_groups;
    double *l2_prev;            // per group
    int32_t *bits;              // per group
    int32_t *counter;           // per group
    uint8_t *rbytes;
    const int64_t *elem_off;
    int64_t *pack_off;
    int32_t *changed;
    int64_t *packed_size;
    int n_layers;
    double T;
    int interval;
    int n_bits;
    int32_t *steps_done;        // 0 before the first batch: that batch only records norms
};

}  // namespace adt
