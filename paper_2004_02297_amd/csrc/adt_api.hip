// C-ABI entry points of libadt (declared in include/adt.h): argument
// validation, per-layer table construction, scratch management, launches.
// All arithmetic of the method on weights happens in the gfx950 kernels; the
// only host arithmetic is on the n_layers-sized tables and the scalar AWP rule.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/adt.h"
#include "../../include/adt_measure.h"
#include "adt_launch.h"
#include "adt_tables.h"
#include "adt_tile_ops.h"

namespace adt {
hipError_t launch_pack(const PackArgs &a, uint32_t n_tiles, bool inline_table, int waves,
                       uint32_t extra_lds, hipStream_t stream);
hipError_t launch_unpack(const PackArgs &a, uint32_t n_tiles, bool inline_table, int out_format,
                         uint32_t extra_lds, hipStream_t stream);
hipError_t launch_stats(const StatsArgs &a, const StatsFinalArgs &f, uint32_t n_tiles,
                        bool inline_table, uint32_t extra_lds, hipStream_t stream);
hipError_t launch_fused(const FusedArgs &a, int out_format, int waves, uint32_t extra_lds,
                        hipStream_t stream);
hipError_t launch_final_rule(const FinalRuleArgs &a, hipStream_t stream);
hipError_t launch_redo(const FusedArgs &a, int out_format, int64_t *pack_off, int64_t *packed_size,
                       int32_t *steps_done, hipStream_t stream);
hipError_t launch_pack_unpack(const PackUnpackArgs &a, uint32_t n_tiles, bool inline_table,
                              int waves, uint32_t extra_lds, hipStream_t stream);
hipError_t launch_ablation(int which, const AblationArgs &a, uint32_t n_tiles, hipStream_t s);
}  // namespace adt

// A plan: device-resident tables + AWP state (see include/adt.h).
struct awp_plan {
    int device = 0;
    int n_layers = 0;
    int n_groups = 0;
    int32_t *group_off = nullptr;
    int64_t n = 0;
    uint32_t n_tiles = 0;
    double T = 0.0;
    int interval = 0, n_bits = 0;
    int64_t steps = 0;
    // Stream bytes per weight as last seen by the host (at creation, set_state
    // and read); only picks the fused kernel's occupancy cap.
    double bytes_per_weight_hint = 1.0;
    hipStream_t last_stream = nullptr;
    std::vector<int64_t> layer_sizes;   // host copy, for rebuilding the stream offsets
    std::vector<int32_t> groups;        // host copy of group_off
    char *block = nullptr;          // one device allocation holding all of the below
    int64_t *elem_off = nullptr, *pack_off = nullptr, *packed_size = nullptr;
    uint32_t *tile_off = nullptr, *partial_absmax = nullptr;
    uint32_t *tile_pivots = nullptr;        // first level of the kernels' tile search
    int pivot_step = 1;
    uint8_t *rbytes = nullptr;
    int32_t *bits = nullptr, *counter = nullptr, *changed = nullptr, *steps_done = nullptr;
    // Leaving the redo launch out (see plan_step): what the fused kernel's first
    // thread keeps on the device, the pinned host word it publishes, and the
    // host's own count of the batches issued since creation / set_state.
    int32_t *rule_seen = nullptr;       // two entries, one per set of partials
    uint32_t *batch_count = nullptr;
    unsigned long long *host_status = nullptr;
    uint32_t issued = 0;
    bool captured = false;      // a step went into a graph: replays are not counted, always redo
    // Two sets of statistics partials.  While no byte count can move, a batch's
    // final reduction and rule are not launched behind its fused kernel but ride
    // at the head of the next batch's fused kernel (or are launched by whoever
    // needs the state first): `pending` says that set `pending_set` waits for that.
    int cur_set = 0, pending_set = 0;
    bool pending = false;
    double *l2_prev = nullptr, *stats = nullptr, *partial_sumsq = nullptr;
    // final reduction + rule: its sub-blocks (see adt::FinalSub) and the slices per chunk
    int n_subs = 0;
    int final_slices = 1;
    adt::FinalSub *subs = nullptr;
    uint32_t *layer_sub_off = nullptr, *sub_absmax = nullptr;
    int32_t *group_subs = nullptr, *group_ticket = nullptr;
    double *sub_sumsq = nullptr;
};

static_assert(ADT_NKERNELS == adt::kNumKernels, "adt.h and adt_launch.h disagree");
static_assert(ADT_OUT_BF16 == adt::kOutBf16 && ADT_OUT_FP16 == adt::kOutFp16,
              "adt.h and adt_tile_ops.h disagree");

// Fixed scratch of awp_layer_stats_noalloc: one double and one magnitude word
// per statistics tile.  Every device the library runs on holds its own copy of
// this array until the process ends; host code reaches a device's copy only
// through the address hipGetSymbolAddress returns for it (noalloc_scratch()).
constexpr uint32_t kNoAllocMaxTiles = AWP_NOALLOC_MAX_TILES;
constexpr size_t kNoAllocScratchBytes = (size_t)kNoAllocMaxTiles * 12;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {

thread_local std::string g_err;

int fail(int status, const std::string &detail) {
    g_err = detail;
    return status;
}

int fail_hip(hipError_t e, const char *what) {
    return fail(ADT_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

// ---- per-device state -----------------------------------------------------
// Large tables (more than adt::kInlineLayers layers) are staged through a
// small ring: pinned host buffer -> device buffer, with an event per slot so
// that a slot is not rewritten while a kernel may still read it.
struct Slot {
    void *host = nullptr;
    void *dev = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};

struct DeviceState {
    Slot ring[4];
    int next = 0;
    void *stats_scratch = nullptr;
    size_t stats_cap = 0;
    // The statistics scratch is shared by all calls on the device: the event
    // marks the end of the last call that used it, and a call on another
    // stream waits for it before it overwrites the partials.
    hipEvent_t stats_ev = nullptr;
    hipStream_t stats_stream = nullptr;
    bool stats_pending = false;
};

std::mutex g_mu;
std::map<int, DeviceState> g_state;

// Launch shape overrides (adt_launch_shape); waves == 0: the library's own choice.
using adt::LaunchShape;
std::mutex g_shape_mu;
LaunchShape g_shape[ADT_NKERNELS] = {};

LaunchShape shape_of(int kernel, LaunchShape dflt) {
    std::lock_guard<std::mutex> lock(g_shape_mu);
    return g_shape[kernel].waves ? g_shape[kernel] : dflt;
}

// Streams above this size are written with nontemporal stores (adt_tile_ops.h):
// one limit for adt_pack, one for the kernels that also write the truncated weights.
std::atomic<int64_t> g_pack_cache_limit{adt::kPackStreamKeepInCacheBytes};
std::atomic<int64_t> g_fused_cache_limit{adt::kFusedStreamKeepInCacheBytes};

// ---- launch timing ----------------------------------------------------------
struct TimedLaunch {
    int kernel;
    hipEvent_t start, stop;
};
std::mutex g_timing_mu;
bool g_timing_on = false;
constexpr size_t kMaxTimedLaunches = 1u << 16;          // launches kept until adt_timing_read
std::vector<TimedLaunch> g_timed;                       // launches not yet read
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_spare;  // event pairs to reuse

bool stream_is_capturing(hipStream_t stream) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

void release_slot(Slot &s) {
    if (s.pending && s.ev) (void)hipEventSynchronize(s.ev);
    if (s.dev) (void)hipFree(s.dev);
    if (s.host) (void)hipHostFree(s.host);
    if (s.ev) (void)hipEventDestroy(s.ev);
    s = Slot();
}

int acquire_slot(DeviceState &st, size_t bytes, Slot **out) {
    Slot &s = st.ring[st.next];
    st.next = (st.next + 1) % 4;
    if (s.pending) {
        hipError_t e = hipEventSynchronize(s.ev);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
        s.pending = false;
    }
    if (!s.ev) {
        hipError_t e = hipEventCreateWithFlags(&s.ev, hipEventDisableTiming);
        if (e != hipSuccess) return fail_hip(e, "hipEventCreate");
    }
    if (s.cap < bytes) {
        if (s.dev) (void)hipFree(s.dev);
        if (s.host) (void)hipHostFree(s.host);
        s.dev = s.host = nullptr;
        s.cap = 0;
        size_t cap = bytes * 2;
        if (hipMalloc(&s.dev, cap) != hipSuccess) {
            (void)hipGetLastError();
            s.dev = nullptr;
            return fail(ADT_ENOMEM, "device table buffer");
        }
        if (hipHostMalloc(&s.host, cap, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(s.dev);
            s.dev = s.host = nullptr;
            return fail(ADT_ENOMEM, "pinned table buffer");
        }
        s.cap = cap;
    }
    *out = &s;
    return ADT_OK;
}

size_t align8(size_t x) { return (x + 7) & ~(size_t)7; }

// Device address of the current device's copy of `scratch`, looked up once per
// device (with that device current) and kept.  No allocation.
constexpr int kMaxDevices = 64;
std::mutex g_noalloc_mu;
unsigned char *g_noalloc_ptr[kMaxDevices] = {};

int noalloc_scratch(unsigned char **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(ADT_ERANGE, "device index out of range");
    std::lock_guard<std::mutex> lock(g_noalloc_mu);
    if (!g_noalloc_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail_hip(e, "hipGetSymbolAddress(scratch)");
        }
        g_noalloc_ptr[dev] = (unsigned char *)p;
    }
    *out = g_noalloc_ptr[dev];
    return ADT_OK;
}

// ---- validation -------------------------------------------------------------
int check_tables(const int64_t *off, const uint8_t *rb, bool need_rb, int n_layers) {
    if (n_layers < 0) return fail(ADT_EINVAL, "n_layers < 0");
    if (!off) return fail(ADT_EINVAL, "layer_offsets is null");
    if (off[0] != 0) return fail(ADT_EINVAL, "layer_offsets[0] != 0");
    if (need_rb && n_layers > 0 && !rb) return fail(ADT_EINVAL, "bytes_per_layer is null");
    for (int l = 0; l < n_layers; ++l) {
        if (off[l + 1] < off[l])
            return fail(ADT_EINVAL, "layer_offsets decreases at layer " + std::to_string(l));
        if (need_rb && (rb[l] < 1 || rb[l] > 4))
            return fail(ADT_EINVAL, "bytes_per_layer[" + std::to_string(l) + "] not in 1..4");
    }
    return ADT_OK;
}

// Tiles per layer -> exclusive prefix; fails if one launch cannot hold them.
int build_tile_off(const int64_t *off, int n_layers, int64_t tile, uint32_t *tile_off) {
    int64_t t = 0;
    for (int l = 0; l < n_layers; ++l) {
        tile_off[l] = (uint32_t)t;
        t += (off[l + 1] - off[l] + tile - 1) / tile;
        if (t >= ((int64_t)1 << 31)) return fail(ADT_ERANGE, "too many tiles for one launch");
    }
    tile_off[n_layers] = (uint32_t)t;
    return ADT_OK;
}

// Groups are runs of consecutive layers; null means one group per layer.
int check_groups(const int32_t *group_offsets, int n_groups, int n_layers,
                 std::vector<int32_t> *out) {
    if (n_groups < 0) return fail(ADT_EINVAL, "n_groups < 0");
    if (!group_offsets) {
        if (n_groups != n_layers)
            return fail(ADT_EINVAL, "without group_offsets n_groups must equal n_layers");
        if (out) {
            out->resize((size_t)n_layers + 1);
            for (int l = 0; l <= n_layers; ++l) (*out)[(size_t)l] = l;
        }
        return ADT_OK;
    }
    if (group_offsets[0] != 0) return fail(ADT_EINVAL, "group_offsets[0] != 0");
    for (int g = 0; g < n_groups; ++g)
        if (group_offsets[g + 1] < group_offsets[g])
            return fail(ADT_EINVAL, "group_offsets decreases");
    if (group_offsets[n_groups] != n_layers)
        return fail(ADT_EINVAL, "group_offsets must end at n_layers");
    if (out) out->assign(group_offsets, group_offsets + n_groups + 1);
    return ADT_OK;
}

enum Direction { kPack, kUnpack, kPackUnpack, kUnpackBf16, kUnpackFp16 };


int pack_or_unpack(Direction dir, const void *weights, const int64_t *off,
                   const uint8_t *rb, int n_layers, const void *packed, adt_stream_t stream,
                   void *weights_out = nullptr) {
    int rc = check_tables(off, rb, true, n_layers);
    if (rc) return rc;
    const int64_t n = n_layers ? off[n_layers] : 0;
    if (n_layers == 0 || n == 0) return ADT_OK;
    if (!weights || !packed) return fail(ADT_EINVAL, "null device pointer");
    const bool out16 = dir == kUnpackBf16 || dir == kUnpackFp16;
    if ((uintptr_t)weights & (out16 ? 1u : 3u))
        return fail(ADT_EALIGN, out16 ? "16-bit buffer is not 2-byte aligned"
                                      : "FP32 buffer is not 4-byte aligned");
    if (dir == kPackUnpack) {
        if (!weights_out) return fail(ADT_EINVAL, "weights_out is null");
        if ((uintptr_t)weights_out & 3u)
            return fail(ADT_EALIGN, "FP32 buffer is not 4-byte aligned");
    }

    adt::PackUnpackArgs pu;
    pu.weights_out = (uint32_t *)weights_out;
    adt::PackArgs &a = pu.p;
    a.weights = (const uint32_t *)weights;
    a.packed = (uint8_t *)packed;
    a.n_layers = n_layers;
    a.stream_cache_limit = dir == kPack ? g_pack_cache_limit.load() : g_fused_cache_limit.load();
    a.dev = adt::DeviceTable{nullptr, nullptr, nullptr, nullptr};
    const bool inl = n_layers <= adt::kInlineLayers;
    hipStream_t hs = (hipStream_t)stream;

    std::unique_lock<std::mutex> lock(g_mu, std::defer_lock);
    Slot *slot = nullptr;
    int64_t *elem_off, *pack_off;
    uint32_t *tile_off;
    uint8_t *rbytes;
    size_t bytes = 0;
    if (inl) {
        elem_off = a.inl.elem_off;
        pack_off = a.inl.pack_off;
        tile_off = a.inl.tile_off;
        rbytes = a.inl.rbytes;
    } else {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
        const size_t L1 = (size_t)n_layers + 1;
        const size_t o_pack = align8(8 * L1), o_tile = o_pack + align8(8 * L1);
        const size_t o_rb = o_tile + align8(4 * L1);
        bytes = o_rb + align8((size_t)n_layers);
        lock.lock();
        rc = acquire_slot(g_state[dev], bytes, &slot);
        if (rc) return rc;
        char *h = (char *)slot->host, *d = (char *)slot->dev;
        elem_off = (int64_t *)h;
        pack_off = (int64_t *)(h + o_pack);
        tile_off = (uint32_t *)(h + o_tile);
        rbytes = (uint8_t *)(h + o_rb);
        a.dev = adt::DeviceTable{(const int64_t *)d, (const int64_t *)(d + o_pack),
                                 (const uint32_t *)(d + o_tile), (const uint8_t *)(d + o_rb)};
    }

    int64_t p = 0;
    for (int l = 0; l < n_layers; ++l) {
        elem_off[l] = off[l];
        pack_off[l] = p;
        rbytes[l] = rb[l];
        p += (off[l + 1] - off[l]) * (int64_t)rb[l];
    }
    elem_off[n_layers] = off[n_layers];
    pack_off[n_layers] = p;
    a.packed_size = p;
    const bool unpack_dir = dir == kUnpack || dir == kUnpackBf16 || dir == kUnpackFp16;
    const double bpw = (double)p / (double)n;            // stream bytes per weight
    const LaunchShape shape =
        dir == kPack ? shape_of(adt::kKernelPack, adt::pack_shape(bpw, p > a.stream_cache_limit))
        : dir == kPackUnpack ? shape_of(adt::kKernelPackUnpack, adt::pack_unpack_shape(bpw))
                             : shape_of(adt::kKernelUnpack, adt::unpack_shape(bpw, dir != kUnpack));
    rc = build_tile_off(off, n_layers,
                        unpack_dir ? adt::kUnpackBlockTile : (int64_t)shape.waves * adt::kWaveTile,
                        tile_off);
    if (rc) return rc;
    const uint32_t n_tiles = tile_off[n_layers];

    if (!inl) {
        hipError_t e = hipMemcpyAsync(slot->dev, slot->host, bytes, hipMemcpyHostToDevice, hs);
        if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync(table)");
    }
    hipError_t e = dir == kPack     ? adt::launch_pack(a, n_tiles, inl, shape.waves, shape.extra_lds, hs)
                   : dir == kUnpack ? adt::launch_unpack(a, n_tiles, inl, 0, shape.extra_lds, hs)
                   : dir == kUnpackBf16
                       ? adt::launch_unpack(a, n_tiles, inl, ADT_OUT_BF16, shape.extra_lds, hs)
                   : dir == kUnpackFp16
                       ? adt::launch_unpack(a, n_tiles, inl, ADT_OUT_FP16, shape.extra_lds, hs)
                                        : adt::launch_pack_unpack(pu, n_tiles, inl, shape.waves,
                                                                  shape.extra_lds, hs);
    if (!inl) {
        // guard the slot even if the launch failed: the copy may be in flight
        if (hipEventRecord(slot->ev, hs) == hipSuccess) slot->pending = true;
        else (void)hipStreamSynchronize(hs);
    }
    if (e != hipSuccess) return fail_hip(e, "pack / unpack launch");
    return ADT_OK;
}

}  // namespace

bool adt::timing_events(int kernel_id, hipStream_t stream, hipEvent_t *start, hipEvent_t *stop) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    if (!g_timing_on) return false;
    if (g_timed.size() >= kMaxTimedLaunches) return false;   // unread records are bounded
    if (stream_is_capturing(stream)) return false;
    std::pair<hipEvent_t, hipEvent_t> ev{nullptr, nullptr};
    if (!g_spare.empty()) {
        ev = g_spare.back();
        g_spare.pop_back();
    } else if (hipEventCreate(&ev.first) != hipSuccess ||
               hipEventCreate(&ev.second) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    g_timed.push_back(TimedLaunch{kernel_id, ev.first, ev.second});
    *start = ev.first;
    *stop = ev.second;
    return true;
}

extern "C" {

int64_t adt_packed_size(const int64_t *layer_offsets, const uint8_t *bytes_per_layer,
                        int n_layers) {
    int rc = check_tables(layer_offsets, bytes_per_layer, true, n_layers);
    if (rc) return rc;
    int64_t p = 0;
    for (int l = 0; l < n_layers; ++l)
        p += (layer_offsets[l + 1] - layer_offsets[l]) * (int64_t)bytes_per_layer[l];
    return p;
}

int adt_pack(const float *weights, const int64_t *layer_offsets,
             const uint8_t *bytes_per_layer, int n_layers, uint8_t *out,
             adt_stream_t stream) {
    return pack_or_unpack(kPack, weights, layer_offsets, bytes_per_layer, n_layers, out, stream);
}

int adt_unpack(const uint8_t *packed, const int64_t *layer_offsets,
               const uint8_t *bytes_per_layer, int n_layers, float *weights_out,
               adt_stream_t stream) {
    return pack_or_unpack(kUnpack, weights_out, layer_offsets, bytes_per_layer, n_layers,
                          packed, stream);
}

int adt_unpack16(const uint8_t *packed, const int64_t *layer_offsets,
                 const uint8_t *bytes_per_layer, int n_layers, uint16_t *out, int format,
                 adt_stream_t stream) {
    if (format != ADT_OUT_BF16 && format != ADT_OUT_FP16)
        return fail(ADT_EINVAL, "format must be ADT_OUT_BF16 or ADT_OUT_FP16");
    return pack_or_unpack(format == ADT_OUT_BF16 ? kUnpackBf16 : kUnpackFp16, out, layer_offsets,
                          bytes_per_layer, n_layers, packed, stream);
}

int adt_pack_unpack(const float *weights, const int64_t *layer_offsets,
                    const uint8_t *bytes_per_layer, int n_layers, uint8_t *out,
                    float *weights_out, adt_stream_t stream) {
    return pack_or_unpack(kPackUnpack, weights, layer_offsets, bytes_per_layer, n_layers, out,
                          stream, weights_out);
}

int awp_layer_stats(const float *weights, const int64_t *layer_offsets, int n_layers,
                    double *stats_out, adt_stream_t stream) {
    int rc = check_tables(layer_offsets, nullptr, false, n_layers);
    if (rc) return rc;
    if (n_layers == 0) return ADT_OK;
    const int64_t n = layer_offsets[n_layers];
    if (!stats_out) return fail(ADT_EINVAL, "stats_out is null");
    if (n > 0 && !weights) return fail(ADT_EINVAL, "weights is null");
    if ((uintptr_t)weights & 3u) return fail(ADT_EALIGN, "FP32 buffer is not 4-byte aligned");
    if ((uintptr_t)stats_out & 7u) return fail(ADT_EALIGN, "stats_out is not 8-byte aligned");

    hipStream_t hs = (hipStream_t)stream;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");

    adt::StatsArgs a;
    adt::StatsFinalArgs f;
    const bool inl = n_layers <= adt::kInlineLayers;
    const size_t L1 = (size_t)n_layers + 1;
    const size_t o_tile = align8(8 * L1);
    const size_t bytes = o_tile + align8(4 * L1);

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState &st = g_state[dev];
    Slot *slot = nullptr;
    int64_t *elem_off;
    uint32_t *tile_off;
    a.dev_elem_off = nullptr;
    a.dev_tile_off = nullptr;
    f.dev_tile_off = nullptr;
    if (inl) {
        elem_off = a.inl.elem_off;
        tile_off = a.inl.tile_off;
    } else {
        rc = acquire_slot(st, bytes, &slot);
        if (rc) return rc;
        elem_off = (int64_t *)slot->host;
        tile_off = (uint32_t *)((char *)slot->host + o_tile);
        a.dev_elem_off = (const int64_t *)slot->dev;
        a.dev_tile_off = (const uint32_t *)((char *)slot->dev + o_tile);
        f.dev_tile_off = a.dev_tile_off;
    }
    for (int l = 0; l <= n_layers; ++l) elem_off[l] = layer_offsets[l];
    rc = build_tile_off(layer_offsets, n_layers, adt::kStatsTile, tile_off);
    if (rc) return rc;
    const uint32_t n_tiles = tile_off[n_layers];
    if (inl) memcpy(f.inl_tile_off, tile_off, 4 * L1);

    // scratch: n_tiles doubles, then n_tiles magnitude words
    const size_t need = (size_t)n_tiles * 12 + 16;
    if (st.stats_cap < need) {
        if (st.stats_scratch) (void)hipFree(st.stats_scratch);   // waits for the device
        st.stats_scratch = nullptr;
        st.stats_cap = 0;
        const size_t cap = need + need / 2 + 4096;
        if (hipMalloc(&st.stats_scratch, cap) != hipSuccess) {
            (void)hipGetLastError();
            st.stats_scratch = nullptr;
            return fail(ADT_ENOMEM, "statistics scratch");
        }
        st.stats_cap = cap;
    }
    a.weights = (const uint32_t *)weights;
    a.partial_sumsq = (double *)st.stats_scratch;
    a.partial_absmax = (uint32_t *)((char *)st.stats_scratch + align8((size_t)n_tiles * 8));
    a.n_layers = n_layers;
    f.partial_sumsq = a.partial_sumsq;
    f.partial_absmax = a.partial_absmax;
    f.stats_out = stats_out;
    f.n_layers = n_layers;

    const bool capturing = stream_is_capturing(hs);
    if (st.stats_pending && st.stats_stream != hs && !capturing) {
        e = hipStreamWaitEvent(hs, st.stats_ev, 0);
        if (e != hipSuccess) return fail_hip(e, "hipStreamWaitEvent(statistics scratch)");
    }
    if (!inl) {
        e = hipMemcpyAsync(slot->dev, slot->host, bytes, hipMemcpyHostToDevice, hs);
        if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync(table)");
    }
    e = adt::launch_stats(a, f, n_tiles, inl,
                          shape_of(adt::kKernelStatsPartial, adt::stats_shape(n_tiles)).extra_lds, hs);
    if (!inl) {
        if (hipEventRecord(slot->ev, hs) == hipSuccess) slot->pending = true;
        else (void)hipStreamSynchronize(hs);
    }
    if (e != hipSuccess) return fail_hip(e, "statistics launch");
    if (!capturing) {
        if (!st.stats_ev &&
            hipEventCreateWithFlags(&st.stats_ev, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            st.stats_ev = nullptr;
        }
        if (st.stats_ev && hipEventRecord(st.stats_ev, hs) == hipSuccess) {
            st.stats_pending = true;
            st.stats_stream = hs;
        } else {
            (void)hipStreamSynchronize(hs);     // no event: fall back to waiting here
            st.stats_pending = false;
        }
    }
    return ADT_OK;
}

int awp_layer_stats_noalloc(const float *weights, const int64_t *layer_offsets, int n_layers,
                            double *stats_out, adt_stream_t stream) {
    int rc = check_tables(layer_offsets, nullptr, false, n_layers);
    if (rc) return rc;
    if (n_layers == 0) return ADT_OK;
    const int64_t n = layer_offsets[n_layers];
    if (!stats_out) return fail(ADT_EINVAL, "stats_out is null");
    if (n > 0 && !weights) return fail(ADT_EINVAL, "weights is null");
    if ((uintptr_t)weights & 3u) return fail(ADT_EALIGN, "FP32 buffer is not 4-byte aligned");
    if ((uintptr_t)stats_out & 7u) return fail(ADT_EALIGN, "stats_out is not 8-byte aligned");
    if (n_layers > adt::kInlineLayers)
        return fail(ADT_ERANGE, "awp_layer_stats_noalloc takes at most " +
                                    std::to_string(adt::kInlineLayers) + " layers");

    adt::StatsArgs a;
    adt::StatsFinalArgs f;
    a.dev_elem_off = nullptr;
    a.dev_tile_off = nullptr;
    f.dev_tile_off = nullptr;
    for (int l = 0; l <= n_layers; ++l) a.inl.elem_off[l] = layer_offsets[l];
    rc = build_tile_off(layer_offsets, n_layers, adt::kStatsTile, a.inl.tile_off);
    if (rc) return rc;
    const uint32_t n_tiles = a.inl.tile_off[n_layers];
    if (n_tiles > kNoAllocMaxTiles)
        return fail(ADT_ERANGE, "awp_layer_stats_noalloc: " + std::to_string(n_tiles) +
                                    " tiles of 8192 weights exceed the fixed scratch of " +
                                    std::to_string(kNoAllocMaxTiles) + " tiles");
    memcpy(f.inl_tile_off, a.inl.tile_off, 4 * ((size_t)n_layers + 1));

    unsigned char *base = nullptr;
    rc = noalloc_scratch(&base);
    if (rc) return rc;
    // Nothing in the scratch has to start at zero: the partial kernel writes
    // every entry [0, n_tiles) that the final kernel reads.
    a.weights = (const uint32_t *)weights;
    a.partial_sumsq = (double *)base;
    a.partial_absmax = (uint32_t *)(base + (size_t)kNoAllocMaxTiles * 8);
    a.n_layers = n_layers;
    f.partial_sumsq = a.partial_sumsq;
    f.partial_absmax = a.partial_absmax;
    f.stats_out = stats_out;
    f.n_layers = n_layers;
    hipError_t e = adt::launch_stats(
        a, f, n_tiles, true, shape_of(adt::kKernelStatsPartial, adt::stats_shape(n_tiles)).extra_lds,
        (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "statistics launch");
    return ADT_OK;
}

int awp_update(const double *l2_now, double *l2_prev, int32_t *counter, int32_t *bits,
               uint8_t *bytes_out, int n_layers, double T, int interval, int n_bits,
               int is_first_batch) {
    if (n_layers < 0) return fail(ADT_EINVAL, "n_layers < 0");
    if (n_layers > 0 && (!l2_now || !l2_prev || !counter || !bits || !bytes_out))
        return fail(ADT_EINVAL, "null state array");
    for (int l = 0; l < n_layers; ++l) {
        if (!is_first_batch) {
            const double prev = l2_prev[l], now = l2_now[l];
            const double delta = prev == 0.0 ? (now == 0.0 ? 0.0 : (double)INFINITY)
                                             : (now - prev) / prev;
            if (delta < T) ++counter[l];
            if (counter[l] == interval) {
                const int32_t b = bits[l] + n_bits;
                bits[l] = b > 32 ? 32 : b;
                counter[l] = 0;
            }
        }
        l2_prev[l] = l2_now[l];
        bytes_out[l] = (uint8_t)((bits[l] + 7) >> 3);
    }
    return ADT_OK;
}

int awp_plan_create(const int64_t *layer_offsets, int n_layers, const int32_t *init_bits,
                    double T, int interval, int n_bits, awp_plan **plan_out) {
    return awp_plan_create_grouped(layer_offsets, n_layers, nullptr, n_layers, init_bits, T,
                                   interval, n_bits, plan_out);
}

int awp_plan_create_grouped(const int64_t *layer_offsets, int n_layers,
                            const int32_t *group_offsets, int n_groups,
                            const int32_t *init_bits, double T, int interval, int n_bits,
                            awp_plan **plan_out) {
    if (!plan_out) return fail(ADT_EINVAL, "plan_out is null");
    *plan_out = nullptr;
    int rc = check_tables(layer_offsets, nullptr, false, n_layers);
    if (rc) return rc;
    if (interval < 1 || n_bits < 0) return fail(ADT_EINVAL, "interval < 1 or n_bits < 0");
    std::vector<int32_t> groups;
    rc = check_groups(group_offsets, n_groups, n_layers, &groups);
    if (rc) return rc;
    const size_t G = (size_t)n_groups;
    const size_t L = (size_t)n_layers, L1 = L + 1;
    std::vector<uint32_t> tile_off(L1);
    rc = build_tile_off(layer_offsets, n_layers, adt::kBlockTile, tile_off.data());
    if (rc) return rc;
    if (tile_off[L] >= (1u << 29)) return fail(ADT_ERANGE, "too many tiles for one launch");
    std::vector<int32_t> bits(G);
    std::vector<uint8_t> rb(L);
    std::vector<int64_t> pack_off(L1);
    for (size_t g = 0; g < G; ++g) {
        const int32_t b = init_bits ? init_bits[g] : 8;
        if (b < 1 || b > 32) return fail(ADT_EINVAL, "init_bits not in 1..32");
        bits[g] = b;
        for (int32_t l = groups[g]; l < groups[g + 1]; ++l) rb[(size_t)l] = (uint8_t)((b + 7) >> 3);
    }
    int64_t p = 0;
    for (size_t l = 0; l < L; ++l) {
        pack_off[l] = p;
        p += (layer_offsets[l + 1] - layer_offsets[l]) * (int64_t)rb[l];
    }
    pack_off[L] = p;

    awp_plan *pl = new (std::nothrow) awp_plan();
    if (!pl) return fail(ADT_ENOMEM, "plan");
    hipError_t e = hipGetDevice(&pl->device);
    if (e != hipSuccess) { delete pl; return fail_hip(e, "hipGetDevice"); }
    pl->n_layers = n_layers;
    pl->n_groups = n_groups;
    pl->groups = groups;
    pl->layer_sizes.resize(L);
    for (size_t l = 0; l < L; ++l) pl->layer_sizes[l] = layer_offsets[l + 1] - layer_offsets[l];
    pl->n = layer_offsets[n_layers];
    pl->bytes_per_weight_hint = pl->n > 0 ? (double)p / (double)pl->n : 1.0;
    pl->n_tiles = tile_off[L];
    pl->T = T;
    pl->interval = interval;
    pl->n_bits = n_bits;

    // sub-blocks of the final reduction + rule: first every layer's chunks in layer
    // order, then one empty sub-block for every group that has no layer
    pl->final_slices = adt::final_slices_for((uint64_t)pl->n_tiles * adt::kWavesPerBlock);
    const uint32_t chunk = (uint32_t)pl->final_slices * adt::kFinalSlice;
    std::vector<adt::FinalSub> subs;
    std::vector<uint32_t> layer_sub_off(L1);
    std::vector<int32_t> group_subs(G, 0);
    for (size_t g = 0; g < G; ++g) {
        for (int32_t l = groups[g]; l < groups[g + 1]; ++l) {
            layer_sub_off[(size_t)l] = (uint32_t)subs.size();
            const uint32_t end = tile_off[(size_t)l + 1] * adt::kWavesPerBlock;
            uint32_t at = tile_off[(size_t)l] * adt::kWavesPerBlock;
            do {
                const uint32_t stop = end - at > chunk ? at + chunk : end;
                subs.push_back(adt::FinalSub{(int32_t)g, l, at, stop});
                ++group_subs[g];
                at = stop;
            } while (at < end);
        }
    }
    layer_sub_off[L] = (uint32_t)subs.size();
    for (size_t g = 0; g < G; ++g) {
        if (group_subs[g] == 0) {
            subs.push_back(adt::FinalSub{(int32_t)g, -1, 0u, 0u});
            group_subs[g] = 1;
        }
    }
    const size_t S = subs.size();
    pl->n_subs = (int)S;

    // carve one allocation (hipMalloc aligns it to 256 bytes); the pivots need 64-byte
    // alignment and go first, then the 8-byte items
    size_t o = 0;
    auto take = [&o](size_t bytes) { size_t at = o; o += align8(bytes); return at; };
    const size_t o_piv = take(64);
    uint32_t pivots[adt::kTilePivots];
    pl->pivot_step = adt::tile_pivots(tile_off.data(), n_layers, pivots);
    const size_t o_elem = take(8 * L1), o_pack = take(8 * L1), o_psize = take(8);
    const size_t n_partials = (size_t)pl->n_tiles * adt::kWavesPerBlock;   // one per wave tile
    const size_t o_prev = take(8 * G), o_stats = take(24 * L), o_psum = take(2 * 8 * n_partials);
    const size_t o_tile = take(4 * L1), o_pmax = take(2 * 4 * n_partials);
    const size_t o_bits = take(4 * G), o_cnt = take(4 * G), o_grp = take(4 * (G + 1));
    const size_t o_chg = take(4), o_steps = take(4), o_rb = take(L);
    const size_t o_seen = take(2 * 4), o_batch = take(4);
    const size_t o_subs = take(sizeof(adt::FinalSub) * S), o_ssum = take(8 * S), o_smax = take(4 * S);
    const size_t o_lso = take(4 * L1), o_gsubs = take(4 * G), o_gtick = take(4 * G);
    const size_t total = o + 8;
    e = hipMalloc((void **)&pl->block, total);
    if (e != hipSuccess) { (void)hipGetLastError(); delete pl; return fail(ADT_ENOMEM, "plan tables"); }
    char *b = pl->block;
    pl->elem_off = (int64_t *)(b + o_elem);
    pl->pack_off = (int64_t *)(b + o_pack);
    pl->packed_size = (int64_t *)(b + o_psize);
    pl->l2_prev = (double *)(b + o_prev);
    pl->stats = (double *)(b + o_stats);
    pl->partial_sumsq = (double *)(b + o_psum);
    pl->tile_off = (uint32_t *)(b + o_tile);
    pl->tile_pivots = (uint32_t *)(b + o_piv);
    pl->partial_absmax = (uint32_t *)(b + o_pmax);
    pl->bits = (int32_t *)(b + o_bits);
    pl->counter = (int32_t *)(b + o_cnt);
    pl->group_off = (int32_t *)(b + o_grp);
    pl->changed = (int32_t *)(b + o_chg);
    pl->steps_done = (int32_t *)(b + o_steps);
    pl->rule_seen = (int32_t *)(b + o_seen);
    pl->batch_count = (uint32_t *)(b + o_batch);
    pl->rbytes = (uint8_t *)(b + o_rb);
    pl->subs = (adt::FinalSub *)(b + o_subs);
    pl->sub_sumsq = (double *)(b + o_ssum);
    pl->sub_absmax = (uint32_t *)(b + o_smax);
    pl->layer_sub_off = (uint32_t *)(b + o_lso);
    pl->group_subs = (int32_t *)(b + o_gsubs);
    pl->group_ticket = (int32_t *)(b + o_gtick);

    // The status word is a convenience: without it every step launches the redo pass.
    if (pl->n_tiles > 0 && n_groups <= adt::kStatusMaxGroups) {
        void *hp = nullptr;
        if (hipHostMalloc(&hp, 8, hipHostMallocDefault) == hipSuccess) {
            pl->host_status = (unsigned long long *)hp;
            *pl->host_status = 0;       // no batch begun, largest counter 0
        } else {
            (void)hipGetLastError();
        }
    }
    e = hipMemset(b, 0, total);
    if (e == hipSuccess) e = hipMemcpy(pl->elem_off, layer_offsets, 8 * L1, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(pl->pack_off, pack_off.data(), 8 * L1, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(pl->packed_size, &p, 8, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(pl->tile_off, tile_off.data(), 4 * L1, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(pl->tile_pivots, pivots, sizeof(pivots), hipMemcpyHostToDevice);
    if (e == hipSuccess && G) e = hipMemcpy(pl->bits, bits.data(), 4 * G, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->group_off, groups.data(), 4 * (G + 1), hipMemcpyHostToDevice);
    if (e == hipSuccess && L) e = hipMemcpy(pl->rbytes, rb.data(), L, hipMemcpyHostToDevice);
    if (e == hipSuccess && S)
        e = hipMemcpy(pl->subs, subs.data(), sizeof(adt::FinalSub) * S, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->layer_sub_off, layer_sub_off.data(), 4 * L1, hipMemcpyHostToDevice);
    if (e == hipSuccess && G)
        e = hipMemcpy(pl->group_subs, group_subs.data(), 4 * G, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(pl->block);
        if (pl->host_status) (void)hipHostFree(pl->host_status);
        delete pl;
        return fail_hip(e, "plan upload");
    }
    *plan_out = pl;
    return ADT_OK;
}

namespace {
int plan_step(awp_plan *plan, const float *weights, uint8_t *packed, int64_t packed_capacity,
              void *weights_out, int out_format, adt_stream_t stream);
}

int awp_adt_step(awp_plan *plan, const float *weights, uint8_t *packed,
                 int64_t packed_capacity, float *weights_out, adt_stream_t stream) {
    return plan_step(plan, weights, packed, packed_capacity, weights_out,
                     weights_out ? adt::kOutFp32 : -1, stream);
}

int awp_adt_step16(awp_plan *plan, const float *weights, uint8_t *packed,
                   int64_t packed_capacity, uint16_t *weights_out, int format,
                   adt_stream_t stream) {
    if (format != ADT_OUT_BF16 && format != ADT_OUT_FP16)
        return fail(ADT_EINVAL, "format must be ADT_OUT_BF16 or ADT_OUT_FP16");
    if (!weights_out) return fail(ADT_EINVAL, "weights_out is null");
    return plan_step(plan, weights, packed, packed_capacity, weights_out, format, stream);
}

namespace {
// Arguments of the final reduction + rule for the batch whose partials are in `set`.
adt::FinalRuleArgs final_rule_args(const awp_plan *plan, int set) {
    const size_t n_partials = (size_t)plan->n_tiles * adt::kWavesPerBlock;
    adt::FinalRuleArgs r;
    r.partial_sumsq = plan->partial_sumsq + (size_t)set * n_partials;
    r.partial_absmax = plan->partial_absmax + (size_t)set * n_partials;
    r.subs = plan->subs;
    r.layer_sub_off = plan->layer_sub_off;
    r.group_subs = plan->group_subs;
    r.group_ticket = plan->group_ticket;
    r.sub_sumsq = plan->sub_sumsq;
    r.sub_absmax = plan->sub_absmax;
    r.stats = plan->stats;
    r.group_off = plan->group_off;
    r.n_subs = plan->n_subs;
    r.n_slices = plan->final_slices;
    r.l2_prev = plan->l2_prev;
    r.bits = plan->bits;
    r.counter = plan->counter;
    r.rbytes = plan->rbytes;
    r.changed = plan->changed;
    // with tiles the fused kernel's first wavefront has set steps_done for the
    // batch already and left the previous value in rule_seen[set]
    r.seen = plan->n_tiles > 0 ? plan->rule_seen + set : plan->steps_done;
    r.T = plan->T;
    r.interval = plan->interval;
    r.n_bits = plan->n_bits;
    return r;
}

// Launches the final reduction + rule of a batch that has been waiting for it.
int flush_pending(awp_plan *plan, hipStream_t hs) {
    if (!plan->pending) return ADT_OK;
    if (stream_is_capturing(hs))
        return fail(ADT_EINVAL,
                    "the last batch's statistics are still to be reduced: call awp_plan_read or "
                    "awp_plan_get_state before capturing on this plan's stream");
    hipError_t e = adt::launch_final_rule(final_rule_args(plan, plan->pending_set), hs);
    if (e != hipSuccess) return fail_hip(e, "final + rule launch");
    plan->pending = false;
    return ADT_OK;
}

int plan_step(awp_plan *plan, const float *weights, uint8_t *packed, int64_t packed_capacity,
              void *weights_out, int out_format, adt_stream_t stream) {
    if (!plan) return fail(ADT_EINVAL, "plan is null");
    hipStream_t hs = (hipStream_t)stream;
    if (plan->n_layers == 0) {
        plan->last_stream = hs;
        return ADT_OK;
    }
    if (plan->n > 0) {
        if (!weights || !packed) return fail(ADT_EINVAL, "null device pointer");
        const bool out16 = out_format == adt::kOutBf16 || out_format == adt::kOutFp16;
        if (((uintptr_t)weights & 3u) || ((uintptr_t)weights_out & (out16 ? 1u : 3u)))
            return fail(ADT_EALIGN, "weight buffer is not aligned to its element size");
        if (packed_capacity < 4 * plan->n)
            return fail(ADT_EINVAL, "packed_capacity must be at least 4 bytes per weight");
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev != plan->device) return fail(ADT_EINVAL, "plan belongs to another device");

    const double out_bytes = out_format == adt::kOutFp32 ? 4.0 : out_format < 0 ? 0.0 : 2.0;
    const LaunchShape shape =
        shape_of(adt::kKernelFused,
                 adt::fused_shape(plan->bytes_per_weight_hint + out_bytes, (int)out_bytes));

    // Can a byte count move in this batch?  Only if the batch takes a group's
    // interval counter to INTERVAL (Algorithm 1).  The status word says how large
    // the largest counter was when some earlier batch began; that batch's
    // predecessor may not have been reduced by then, and every batch issued since
    // adds at most one.  If even that bound stays below INTERVAL - 1, nothing can
    // move: the redo pass has nothing to do and this batch's final reduction and
    // rule need not run before the next batch starts.  A stale or never-updated
    // word only makes the bound larger.  Under graph capture the choice would be
    // frozen into the graph and replays are not counted here: a plan that has
    // been captured takes the in-order path from then on.
    bool quiet = false;
    if (plan->host_status && !plan->captured) {
        if (stream_is_capturing(hs)) {
            plan->captured = true;
        } else {
            const unsigned long long word = __atomic_load_n(plan->host_status, __ATOMIC_RELAXED);
            const uint32_t begun = (uint32_t)(word >> 32), top = (uint32_t)word;
            const uint32_t reduced = begun > 0u ? begun - 1u : 0u;
            const uint64_t bound = (uint64_t)top + (uint32_t)(plan->issued - reduced);
            quiet = bound + 1 < (uint64_t)plan->interval;
        }
    }
    const bool carry = quiet && shape.waves == 1;    // one-wave blocks can carry sub-blocks
    if (!carry) {
        const int rc = flush_pending(plan, hs);      // in order from here on
        if (rc) return rc;
    }
    plan->last_stream = hs;

    const int set = plan->cur_set;
    const size_t n_partials = (size_t)plan->n_tiles * adt::kWavesPerBlock;
    adt::FusedArgs a;
    a.weights = (const uint32_t *)weights;
    a.packed = packed;
    a.weights_out = weights_out;
    a.elem_off = plan->elem_off;
    a.pack_off = plan->pack_off;
    a.tile_off = plan->tile_off;
    a.tile_pivots = plan->tile_pivots;
    a.pivot_step = plan->pivot_step;
    a.rbytes = plan->rbytes;
    a.partial_sumsq = plan->partial_sumsq + (size_t)set * n_partials;
    a.partial_absmax = plan->partial_absmax + (size_t)set * n_partials;
    a.changed = plan->changed;
    a.steps_done = plan->steps_done;
    a.rule_seen = plan->rule_seen + set;
    a.batch_count = plan->batch_count;
    a.counter = plan->counter;
    a.n_status_groups = plan->host_status ? plan->n_groups : 0;
    a.host_status = plan->host_status;
    a.stream_cache_limit = g_fused_cache_limit.load();
    a.n_layers = plan->n_layers;
    a.n_tiles = plan->n_tiles;
    a.n_pending_subs = 0;
    a.pending = final_rule_args(plan, plan->pending_set);
    if (carry && plan->pending) a.n_pending_subs = (uint32_t)plan->n_subs;

    if (plan->n_tiles > 0) {
        e = adt::launch_fused(a, out_format, shape.waves, shape.extra_lds, hs);
        if (e != hipSuccess) return fail_hip(e, "fused launch");
    }
    ++plan->steps;
    ++plan->issued;
    plan->cur_set = set ^ 1;
    if (carry) {
        // this batch's reduction rides with the next batch (or is launched by
        // whoever needs the state first)
        plan->pending = true;
        plan->pending_set = set;
        return ADT_OK;
    }
    plan->pending = false;
    if (plan->n_subs > 0) {
        e = adt::launch_final_rule(final_rule_args(plan, set), hs);
        if (e != hipSuccess) return fail_hip(e, "final + rule launch");
    }
    if (!quiet) {
        e = adt::launch_redo(a, out_format, plan->pack_off, plan->packed_size, plan->steps_done, hs);
        if (e != hipSuccess) return fail_hip(e, "redo launch");
    }
    return ADT_OK;
}
}  // namespace

int awp_plan_flush(awp_plan *plan) {
    if (!plan) return fail(ADT_EINVAL, "plan is null");
    return flush_pending(plan, plan->last_stream);
}

int awp_plan_read(awp_plan *plan, double *stats, int32_t *bits, int32_t *counter,
                  uint8_t *bytes, int64_t *packed_size) {
    if (!plan) return fail(ADT_EINVAL, "plan is null");
    hipStream_t hs = plan->last_stream;
    const int rc = flush_pending(plan, hs);
    if (rc) return rc;
    const size_t L = (size_t)plan->n_layers;
    hipError_t e = hipSuccess;
    auto get = [&](void *dst, const void *src, size_t bytes_) {
        if (dst && bytes_ && e == hipSuccess)
            e = hipMemcpyAsync(dst, src, bytes_, hipMemcpyDeviceToHost, hs);
    };
    get(stats, plan->stats, 24 * L);
    get(bits, plan->bits, 4 * (size_t)plan->n_groups);
    get(counter, plan->counter, 4 * (size_t)plan->n_groups);
    get(bytes, plan->rbytes, L);
    int64_t size_now = 0;
    get(&size_now, plan->packed_size, 8);
    if (e == hipSuccess) e = hipStreamSynchronize(hs);
    if (e != hipSuccess) return fail_hip(e, "plan read");
    if (packed_size) *packed_size = size_now;
    if (plan->n > 0) plan->bytes_per_weight_hint = (double)size_now / (double)plan->n;
    return ADT_OK;
}

int awp_plan_get_state(awp_plan *plan, int32_t *bits, int32_t *counter, double *l2_prev,
                       int32_t *batches_seen) {
    if (!plan) return fail(ADT_EINVAL, "plan is null");
    hipStream_t hs = plan->last_stream;
    const int rc = flush_pending(plan, hs);
    if (rc) return rc;
    const size_t G = (size_t)plan->n_groups;
    hipError_t e = hipSuccess;
    auto get = [&](void *dst, const void *src, size_t n) {
        if (dst && n && e == hipSuccess) e = hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToHost, hs);
    };
    get(bits, plan->bits, 4 * G);
    get(counter, plan->counter, 4 * G);
    get(l2_prev, plan->l2_prev, 8 * G);
    get(batches_seen, plan->steps_done, 4);
    if (e == hipSuccess) e = hipStreamSynchronize(hs);
    if (e != hipSuccess) return fail_hip(e, "plan get_state");
    return ADT_OK;
}

int awp_plan_set_state(awp_plan *plan, const int32_t *bits, const int32_t *counter,
                       const double *l2_prev, int32_t batches_seen) {
    if (!plan) return fail(ADT_EINVAL, "plan is null");
    const size_t G = (size_t)plan->n_groups, L = (size_t)plan->n_layers;
    if (G && (!bits || !counter || !l2_prev)) return fail(ADT_EINVAL, "null state array");
    std::vector<uint8_t> rb(L);
    std::vector<int64_t> pack_off(L + 1);
    for (size_t g = 0; g < G; ++g) {
        if (bits[g] < 1 || bits[g] > 32) return fail(ADT_EINVAL, "bits not in 1..32");
        if (counter[g] < 0) return fail(ADT_EINVAL, "negative counter");
        for (int32_t l = plan->groups[g]; l < plan->groups[g + 1]; ++l)
            rb[(size_t)l] = (uint8_t)((bits[g] + 7) >> 3);
    }
    int64_t p = 0;
    for (size_t l = 0; l < L; ++l) {
        pack_off[l] = p;
        p += plan->layer_sizes[l] * (int64_t)rb[l];
    }
    pack_off[L] = p;
    const int32_t seen = batches_seen != 0;
    const int rc = flush_pending(plan, plan->last_stream);    // its results are replaced below
    if (rc) return rc;
    hipError_t e = hipStreamSynchronize(plan->last_stream);   // earlier steps still read the tables
    auto put = [&](void *dst, const void *src, size_t n) {
        if (n && e == hipSuccess) e = hipMemcpy(dst, src, n, hipMemcpyHostToDevice);
    };
    put(plan->bits, bits, 4 * G);
    put(plan->counter, counter, 4 * G);
    put(plan->l2_prev, l2_prev, 8 * G);
    put(plan->rbytes, rb.data(), L);
    put(plan->pack_off, pack_off.data(), 8 * (L + 1));
    put(plan->packed_size, &p, 8);
    put(plan->steps_done, &seen, 4);
    int32_t top = 0;                            // the counting of batches starts over
    for (size_t g = 0; g < G; ++g) top = counter[g] > top ? counter[g] : top;
    const uint32_t zero = 0;
    put(plan->batch_count, &zero, 4);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess && plan->host_status) {
        __atomic_store_n(plan->host_status, (unsigned long long)(uint32_t)top, __ATOMIC_RELAXED);
        plan->issued = 0;
    }
    if (e != hipSuccess) return fail_hip(e, "plan set_state");
    if (plan->n > 0) plan->bytes_per_weight_hint = (double)p / (double)plan->n;
    return ADT_OK;
}

int awp_plan_destroy(awp_plan *plan) {
    if (!plan) return ADT_OK;
    if (plan->block) {
        int saved = 0;
        const bool have = hipGetDevice(&saved) == hipSuccess;
        if (hipSetDevice(plan->device) == hipSuccess) {
            (void)hipFree(plan->block);   // waits
            if (plan->host_status) (void)hipHostFree(plan->host_status);
        }
        if (have) (void)hipSetDevice(saved);
    }
    delete plan;
    return ADT_OK;
}

int adt_ablation(int variant, int unpack, const float *weights, const int64_t *layer_offsets,
                 const uint8_t *bytes_per_layer, int n_layers, uint8_t *packed,
                 adt_stream_t stream) {
    int rc = check_tables(layer_offsets, bytes_per_layer, true, n_layers);
    if (rc) return rc;
    const int64_t n = n_layers ? layer_offsets[n_layers] : 0;
    if (n_layers == 0 || n == 0) return ADT_OK;
    if (!weights || !packed) return fail(ADT_EINVAL, "null device pointer");
    if ((uintptr_t)weights & 3u) return fail(ADT_EALIGN, "FP32 buffer is not 4-byte aligned");
    hipStream_t hs = (hipStream_t)stream;

    if (variant == ADT_ABLATION_PER_LAYER) {
        int64_t p = 0;
        for (int l = 0; l < n_layers; ++l) {
            const int64_t two[2] = {0, layer_offsets[l + 1] - layer_offsets[l]};
            rc = pack_or_unpack(unpack ? kUnpack : kPack, weights + layer_offsets[l], two,
                                bytes_per_layer + l, 1, packed + p, stream);
            if (rc) return rc;
            p += two[1] * (int64_t)bytes_per_layer[l];
        }
        return ADT_OK;
    }
    if (variant != ADT_ABLATION_NAIVE && variant != ADT_ABLATION_VEC_DIRECT)
        return fail(ADT_EINVAL, "unknown ablation variant");
    if (variant == ADT_ABLATION_VEC_DIRECT && unpack)
        return fail(ADT_EINVAL, "the direct-store variant exists for pack only");
    if (n_layers > adt::kInlineLayers) return fail(ADT_ERANGE, "ablation kernels take <= 128 layers");

    adt::AblationArgs a;
    a.weights = (const uint32_t *)weights;
    a.packed = packed;
    a.n_layers = n_layers;
    const int64_t tile = variant == ADT_ABLATION_NAIVE ? adt::kNaiveTile : adt::kVecTile;
    int64_t p = 0;
    for (int l = 0; l < n_layers; ++l) {
        a.elem_off[l] = layer_offsets[l];
        a.pack_off[l] = p;
        a.rbytes[l] = bytes_per_layer[l];
        if (variant == ADT_ABLATION_VEC_DIRECT &&
            ((((uintptr_t)packed + (uintptr_t)p) & 3u) || (layer_offsets[l] & 3)))
            return fail(ADT_EALIGN, "direct-store variant needs 4-byte aligned layer starts");
        p += (layer_offsets[l + 1] - layer_offsets[l]) * (int64_t)bytes_per_layer[l];
    }
    a.elem_off[n_layers] = layer_offsets[n_layers];
    a.pack_off[n_layers] = p;
    rc = build_tile_off(layer_offsets, n_layers, tile, a.tile_off);
    if (rc) return rc;
    const int which = variant == ADT_ABLATION_NAIVE ? (unpack ? 1 : 0) : 2;
    hipError_t e = adt::launch_ablation(which, a, a.tile_off[n_layers], hs);
    if (e != hipSuccess) return fail_hip(e, "ablation launch");
    return ADT_OK;
}

int awp_group_norms(const double *stats, const int32_t *group_offsets, int n_groups,
                    double *l2_group) {
    if (n_groups < 0 || !group_offsets || (n_groups > 0 && (!stats || !l2_group)))
        return fail(ADT_EINVAL, "null argument or n_groups < 0");
    int rc = check_groups(group_offsets, n_groups, group_offsets[n_groups], nullptr);
    if (rc) return rc;
    for (int g = 0; g < n_groups; ++g) {
        double sumsq = 0.0;
        for (int32_t l = group_offsets[g]; l < group_offsets[g + 1]; ++l)
            sumsq += stats[(size_t)l * AWP_NSTATS + AWP_STAT_SUMSQ];
        l2_group[g] = sqrt(sumsq);
    }
    return ADT_OK;
}

int awp_expand_group_bytes(const uint8_t *bytes_group, const int32_t *group_offsets,
                           int n_groups, uint8_t *bytes_layer) {
    if (n_groups < 0 || !group_offsets || (n_groups > 0 && (!bytes_group || !bytes_layer)))
        return fail(ADT_EINVAL, "null argument or n_groups < 0");
    int rc = check_groups(group_offsets, n_groups, group_offsets[n_groups], nullptr);
    if (rc) return rc;
    for (int g = 0; g < n_groups; ++g)
        for (int32_t l = group_offsets[g]; l < group_offsets[g + 1]; ++l)
            bytes_layer[l] = bytes_group[g];
    return ADT_OK;
}

const char *adt_strerror(int status) {
    switch (status) {
        case ADT_OK: return "success";
        case ADT_EINVAL: return "invalid argument";
        case ADT_EALIGN: return "misaligned buffer";
        case ADT_EHIP: return "HIP runtime error";
        case ADT_ENOMEM: return "out of memory";
        case ADT_ERANGE: return "size out of range";
        default: return "unknown status";
    }
}

const char *adt_last_error(void) { return g_err.c_str(); }

#ifndef ADT_SOURCE_DIGEST
#define ADT_SOURCE_DIGEST ""
#endif
// The marker lets a loader find the digest in the file's bytes without mapping
// the library (a library once mapped stays mapped under its path).
static const char kSourceDigest[] = "adt-source-digest:" ADT_SOURCE_DIGEST;
const char *adt_source_digest(void) { return kSourceDigest + sizeof("adt-source-digest:") - 1; }

int64_t adt_stream_cache_limit(int kernel, int64_t bytes) {
    std::atomic<int64_t> *limit = kernel == adt::kKernelPack ? &g_pack_cache_limit
                                  : kernel == adt::kKernelPackUnpack || kernel == adt::kKernelFused
                                      ? &g_fused_cache_limit
                                      : nullptr;
    if (!limit) return fail(ADT_EINVAL, "stream cache limit: kernel must be pack, pack_unpack or fused");
    if (bytes < 0) return limit->load();
    return limit->exchange(bytes);
}

int adt_launch_shape(int kernel, int waves, int extra_lds_bytes) {
    const bool ok_kernel = kernel == adt::kKernelPack || kernel == adt::kKernelPackUnpack ||
                           kernel == adt::kKernelFused || kernel == adt::kKernelUnpack ||
                           kernel == adt::kKernelStatsPartial;
    if (!ok_kernel)
        return fail(ADT_EINVAL,
                    "launch shape: kernel must be pack, unpack, pack_unpack, fused or stats_partial");
    const bool ok_waves = waves == 0 || (waves == 1 && kernel != adt::kKernelStatsPartial) ||
                          (waves == 4 && kernel != adt::kKernelUnpack);
    if (!ok_waves)
        return fail(ADT_EINVAL, "launch shape: waves must be 0, 1 or 4 (unpack: 1, stats_partial: 4)");
    if (extra_lds_bytes < 0 || extra_lds_bytes > 60 * 1024)
        return fail(ADT_EINVAL, "launch shape: extra LDS must be within 0..60 KiB");
    std::lock_guard<std::mutex> lock(g_shape_mu);
    g_shape[kernel] = LaunchShape{waves, (uint32_t)extra_lds_bytes};
    return ADT_OK;
}

int adt_timing_enable(int on, int reserve_launches) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    g_timing_on = on != 0;
    while (on && (int)g_spare.size() < reserve_launches) {
        std::pair<hipEvent_t, hipEvent_t> ev{nullptr, nullptr};
        hipError_t e = hipEventCreate(&ev.first);
        if (e == hipSuccess) e = hipEventCreate(&ev.second);
        if (e != hipSuccess) return fail_hip(e, "hipEventCreate");
        g_spare.push_back(ev);
    }
    return ADT_OK;
}

int adt_timing_read(adt_kernel_time *out) {
    if (!out) return fail(ADT_EINVAL, "out is null");
    std::lock_guard<std::mutex> lock(g_timing_mu);
    for (int k = 0; k < ADT_NKERNELS; ++k) out[k] = adt_kernel_time{0, 0.0, 0.0, 0.0};
    int rc = ADT_OK;
    for (const TimedLaunch &t : g_timed) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(t.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.start, t.stop);
        if (e != hipSuccess) {
            rc = fail_hip(e, "launch timing");
        } else if (t.kernel >= 0 && t.kernel < ADT_NKERNELS) {
            adt_kernel_time &o = out[t.kernel];
            o.min_ms = o.launches == 0 || ms < o.min_ms ? ms : o.min_ms;
            o.max_ms = ms > o.max_ms ? ms : o.max_ms;
            o.total_ms += ms;
            ++o.launches;
        }
        g_spare.emplace_back(t.start, t.stop);
    }
    g_timed.clear();
    return rc;
}

const char *adt_kernel_name(int kernel) {
    switch (kernel) {
        case adt::kKernelPack: return "pack_kernel";
        case adt::kKernelUnpack: return "unpack_kernel";
        case adt::kKernelStatsPartial: return "stats_partial_kernel";
        case adt::kKernelStatsFinal: return "stats_final_kernel";
        case adt::kKernelFused: return "fused_kernel";
        case adt::kKernelFinalRule: return "final_rule_kernel";
        case adt::kKernelRedo: return "redo_kernel";
        case adt::kKernelPackUnpack: return "pack_unpack_kernel";
        case adt::kKernelUnpack16: return "unpack16_kernel";
        case adt::kKernelPrefix: return "prefix_kernel";
        default: return "";
    }
}

int adt_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int saved = 0;
    const bool have = hipGetDevice(&saved) == hipSuccess;
    for (auto &kv : g_state) {
        if (hipSetDevice(kv.first) != hipSuccess) continue;
        for (Slot &s : kv.second.ring) release_slot(s);
        if (kv.second.stats_scratch) (void)hipFree(kv.second.stats_scratch);
        if (kv.second.stats_ev) (void)hipEventDestroy(kv.second.stats_ev);
    }
    g_state.clear();
    if (have) (void)hipSetDevice(saved);
    {
        std::lock_guard<std::mutex> tlock(g_timing_mu);
        g_timing_on = false;
        for (const TimedLaunch &t : g_timed) g_spare.emplace_back(t.start, t.stop);
        g_timed.clear();
        for (auto &ev : g_spare) {
            (void)hipEventDestroy(ev.first);
            (void)hipEventDestroy(ev.second);
        }
        g_spare.clear();
    }
    return ADT_OK;
}

}  // extern "C"
