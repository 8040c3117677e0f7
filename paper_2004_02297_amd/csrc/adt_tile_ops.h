// Device-side building blocks shared by the ADT kernels (gfx950): cache-hinted
// 128-bit accesses, the byte selection of Bitpack / Bitunpack (Section III,
// Algorithms 2 and 5 of arXiv 2004.02297) on four weights at a time, and the
// wave-tile movers that stage the byte stream through a wave-private LDS slice.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_tables.h"

namespace adt {


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));   // FP32 side: dword aligned

// Cache hints.  FP32 weights are read once by pack and written once by unpack,
// and the stream is read once by unpack: those accesses carry the nontemporal
// hint, so their lines are not kept in L2 / Infinity Cache (on MI355X this
// raises the sustained read rate by about 10 %).  How the stream is WRITTEN
// depends on who reads it next.  Measured on 138 M weights with rotating output
// buffers (so that a rewrite of the same buffer cannot be absorbed by the
// 256 MB Infinity Cache):
//  - adt_pack with adt_unpack right behind it: ordinary stream stores let
//    unpack find much of the stream in the cache.  pack + unpack at 2 bytes
//    (264 MiB stream) 238 us vs 257 us with nontemporal stores, mixed bytes
//    (295 MiB) 249 vs 269 us, 3 bytes (396 MiB) 313 vs 309 us: ordinary stores
//    up to 320 MiB, nontemporal above.
//  - the kernels that also write the truncated weights (adt_pack_unpack, the
//    plan's fused kernel): nothing on the device reads the stream right behind
//    them (a device-to-device copy of the stream placed there runs equally fast
//    either way), and nontemporal stores are 2 - 5 % faster at every size
//    (2 bytes: 218 vs 224 us, 4 bytes: 261 vs 274 us): always nontemporal.
// A streaming store carries two cache-policy bits of the gfx940 family: `nt`
// (nontemporal) and `sc1` (written through at device scope instead of staying
// dirty in the L2 of the XCD).  With all of a wave's stores issued together at
// its end, `sc1 nt` is 2 - 3 % faster than `nt` alone for the write-heavy
// kernels (fused kernel at 2 bytes: 212 vs 217 us; `sc1` without `nt` is slower
// than either).  The compiler sets `nt` for a nontemporal store and `sc1` for an
// agent-scope atomic, but has no way to set both on a 128-bit store, so the
// instruction is written out.  The gfx940 family needs two wait states before
// a later VALU instruction may overwrite the data registers of a store wider
// than 64 bits; the compiler keeps them for its own stores but does not look
// into an asm statement, hence the s_nop 1 (= two wait states) behind the store.
constexpr int64_t kPackStreamKeepInCacheBytes = (int64_t)320 << 20;
constexpr int64_t kFusedStreamKeepInCacheBytes = 0;

#ifndef ADT_NT_FP32_LOAD
#define ADT_NT_FP32_LOAD 1
#endif
#ifndef ADT_NT_FP32_STORE
#define ADT_NT_FP32_STORE 1
#endif
#ifndef ADT_NT_STREAM_LOAD
#define ADT_NT_STREAM_LOAD 1
#endif
__device__ __forceinline__ u32x4 load_fp32x4(const uint32_t *p) {
    if (ADT_NT_FP32_LOAD) return __builtin_nontemporal_load((const u32x4_a4 *)p);
    return *(const u32x4_a4 *)p;
}
__device__ __forceinline__ void store_streaming16(void *p, const u32x4 v) {   // p: 4-byte aligned
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_fp32x4(uint32_t *p, const u32x4 v) {
    if (ADT_NT_FP32_STORE) store_streaming16(p, v);
    else *(u32x4_a4 *)p = v;
}
__device__ __forceinline__ u32x4 load_stream16(const uint8_t *p) {   // 16-byte aligned
    if (ADT_NT_STREAM_LOAD) return __builtin_nontemporal_load((const u32x4 *)p);
    return *(const u32x4 *)p;
}
__device__ __forceinline__ void store_stream16(uint8_t *p, const u32x4 v, bool nt) {
    if (nt) {                                   // nt is wave uniform
        store_streaming16(p, v);
    } else {
        *(u32x4 *)p = v;
    }
}

constexpr int kPadDw = 8;                              // LDS pad before / after
constexpr int kWaveLdsDw = kPadDw + kWaveTile + kPadDw;  // 1040 dwords per wave
constexpr int kPadBytes = kPadDw * 4;

__device__ __forceinline__ void wave_lds_sync() {
    // LDS traffic of one wave is served in order; this only stops the
    // compiler from moving accesses across the exchange point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ({hi,lo} >> 8*sh) truncated to 32 bits, sh in 0..3.
__device__ __forceinline__ uint32_t funnel(uint32_t hi, uint32_t lo, uint32_t sh) {
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> (8u * sh));
}

// Top R bytes of four words, as R dwords of stream (low kept byte first).
template <int R>
__device__ __forceinline__ void keep_top_bytes(const u32x4 u, uint32_t *d) {
    if (R == 4) {
        d[0] = u.x; d[1] = u.y; d[2] = u.z; d[3] = u.w;
    } else if (R == 3) {
        d[0] = (u.x >> 8) | ((u.y >> 8) << 24);
        d[1] = (u.y >> 16) | ((u.z >> 8) << 16);
        d[2] = (u.z >> 24) | ((u.w >> 8) << 8);
    } else if (R == 2) {
        d[0] = (u.x >> 16) | (u.y & 0xFFFF0000u);
        d[1] = (u.z >> 16) | (u.w & 0xFFFF0000u);
    } else {
        d[0] = (u.x >> 24) | ((u.y >> 24) << 8) | ((u.z >> 24) << 16) |
               (u.w & 0xFF000000u);
    }
}

// Inverse: R dwords of stream -> four words with the low 8*(4-R) bits zero.
template <int R>
__device__ __forceinline__ u32x4 shift_to_top(const uint32_t *y) {
    u32x4 u;
    if (R == 4) {
        u.x = y[0]; u.y = y[1]; u.z = y[2]; u.w = y[3];
    } else if (R == 3) {
        u.x = y[0] << 8;
        u.y = ((y[0] >> 24) | (y[1] << 8)) << 8;
        u.z = ((y[1] >> 16) | (y[2] << 16)) << 8;
        u.w = y[2] & 0xFFFFFF00u;
    } else if (R == 2) {
        u.x = y[0] << 16;
        u.y = y[0] & 0xFFFF0000u;
        u.z = y[1] << 16;
        u.w = y[1] & 0xFFFF0000u;
    } else {
        u.x = y[0] << 24;
        u.y = (y[0] << 16) & 0xFF000000u;
        u.z = (y[0] << 8) & 0xFF000000u;
        u.w = y[0] & 0xFF000000u;
    }
    return u;
}

__device__ __forceinline__ uint32_t byte_of(const u32x4 v, int t) {
    uint32_t w = (t < 8) ? ((t < 4) ? v.x : v.y) : ((t < 12) ? v.z : v.w);
    return (w >> (8 * (t & 3))) & 0xFFu;
}

// ---------------------------------------------------------------------------
// Load one wave tile: `len` (1..1024) FP32 words at src, four 128-bit loads per
// lane; lane holds words 4c..4c+3 of the tile for c = j*64 + lane.  Words past
// `len` read as zero.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void load_wave_tile(const uint32_t *__restrict__ src, int len,
                                               int lane, u32x4 (&v)[kChunksPerLane]) {
    if (len == kWaveTile) {
#pragma unroll
        for (int j = 0; j < kChunksPerLane; ++j)
            v[j] = load_fp32x4(src + 4 * (j * kWave + lane));
    } else {
#pragma unroll
        for (int j = 0; j < kChunksPerLane; ++j) {
            const int e0 = 4 * (j * kWave + lane);
            u32x4 t = {0u, 0u, 0u, 0u};
            if (e0 + 4 <= len) {
                t = load_fp32x4(src + e0);
            } else {
                if (e0 < len) t.x = src[e0];
                if (e0 + 1 < len) t.y = src[e0 + 1];
                if (e0 + 2 < len) t.z = src[e0 + 2];
            }
            v[j] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// Write the top R bytes of a loaded wave tile as len*R stream bytes at dst.
// lds: this wave's slice (kWaveLdsDw dwords).
// ---------------------------------------------------------------------------
template <int R>
__device__ __forceinline__ void stream_out_wave_tile(const u32x4 (&v)[kChunksPerLane],
                                                     uint8_t *__restrict__ dst, int len,
                                                     uint32_t *lds, int lane, bool stream_nt) {
    uint32_t *body = lds + kPadDw;
    const uint32_t s = (uint32_t)((uintptr_t)dst & 15u);   // wave uniform
#pragma unroll
    for (int j = 0; j < kChunksPerLane; ++j) {
        uint32_t d[4];
        keep_top_bytes<R>(v[j], d);
        uint32_t *p = body + (j * kWave + lane) * R;
#pragma unroll
        for (int t = 0; t < R; ++t) p[t] = d[t];
    }
    wave_lds_sync();

    if (len == kWaveTile && s == 0) {
        // stream side 16-byte aligned: R full-width stores per lane
#pragma unroll
        for (int k = 0; k < R * kChunksPerLane / 4; ++k) {
            const int q = k * kWave + lane;
            const u32x4 o = *(const u32x4 *)(body + 4 * q);
            store_stream16(dst + 16 * q, o, stream_nt);
        }
        return;
    }

    // General case: walk the 16-byte grid of absolute stream addresses.
    // Piece q covers tile-local stream bytes [16q - s, 16q - s + 16).
    const int nbytes = len * R;
    uint8_t *dst_al = dst - s;
    const int npieces = (int)(s + nbytes + 15) >> 4;
    const uint32_t sh = (0u - s) & 3u;
    for (int k = 0; k * kWave < npieces; ++k) {
        const int q = k * kWave + lane;
        if (q < npieces) {
            const int b0 = 16 * q - (int)s;
            const int dw = (kPadBytes + b0) >> 2;          // >= 4, <= kWaveTile + 7
            const uint32_t x0 = lds[dw], x1 = lds[dw + 1], x2 = lds[dw + 2],
                           x3 = lds[dw + 3], x4 = lds[dw + 4];
            u32x4 o;
            o.x = funnel(x1, x0, sh);
            o.y = funnel(x2, x1, sh);
            o.z = funnel(x3, x2, sh);
            o.w = funnel(x4, x3, sh);
            if (b0 >= 0 && b0 + 16 <= nbytes) {
                store_stream16(dst_al + 16 * q, o, stream_nt);
            } else {
                for (int t = 0; t < 16; ++t) {
                    const int bt = b0 + t;
                    if (bt >= 0 && bt < nbytes) dst_al[16 * q + t] = (uint8_t)byte_of(o, t);
                }
            }
        }
    }
}

// Pack one wave tile: `len` (1..1024) FP32 words at src -> len*R bytes at dst.
template <int R>
__device__ __forceinline__ void pack_wave_tile(const uint32_t *__restrict__ src,
                                               uint8_t *__restrict__ dst, int len,
                                               uint32_t *lds, int lane, bool stream_nt) {
    u32x4 v[kChunksPerLane];
    load_wave_tile(src, len, lane, v);
    stream_out_wave_tile<R>(v, dst, len, lds, lane, stream_nt);
}

// ---------------------------------------------------------------------------
// Output formats of unpack: the FP32 word of Algorithm 5, or a 16-bit compute
// format made from it (the combination with mixed-precision training that the
// paper's related-work section proposes).
// ---------------------------------------------------------------------------
constexpr int kOutFp32 = 0;
constexpr int kOutBf16 = 1;   // top 16 bits of the word (truncation, like ADT itself)
constexpr int kOutFp16 = 2;   // binary16, round to nearest even, overflow to infinity, NaN -> 0x7E00 | sign

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));

template <int OUT>
__device__ __forceinline__ uint32_t to_half_bits(uint32_t word) {
    if (OUT == kOutBf16) return word >> 16;
    const uint32_t half = (uint32_t)__half_as_ushort(__float2half_rn(__uint_as_float(word)));
    const bool is_nan = (word & 0x7FFFFFFFu) > 0x7F800000u;
    return is_nan ? (((word >> 16) & 0x8000u) | 0x7E00u) : half;   // one NaN, sign kept
}

// Store the four unpacked words of chunk starting at tile element e0.
// dst: tile start; FP32 (4-byte aligned) or 16-bit elements (2-byte aligned).
template <int OUT>
__device__ __forceinline__ void store_unpacked(void *dst, int e0, int len, const u32x4 u,
                                               bool dst_dword_aligned) {
    if (OUT == kOutFp32) {
        uint32_t *d = (uint32_t *)dst;
        if (e0 + 4 <= len) {
            store_fp32x4(d + e0, u);
        } else {
            d[e0] = u.x;
            if (e0 + 1 < len) d[e0 + 1] = u.y;
            if (e0 + 2 < len) d[e0 + 2] = u.z;
        }
    } else {
        uint16_t *d = (uint16_t *)dst;
        const uint32_t h0 = to_half_bits<OUT>(u.x), h1 = to_half_bits<OUT>(u.y),
                       h2 = to_half_bits<OUT>(u.z), h3 = to_half_bits<OUT>(u.w);
        if (e0 + 4 <= len && dst_dword_aligned) {
            u32x2 o;
            o.x = h0 | (h1 << 16);
            o.y = h2 | (h3 << 16);
            __builtin_nontemporal_store(o, (u32x2_a4 *)(d + e0));
        } else {
            if (e0 < len) d[e0] = (uint16_t)h0;
            if (e0 + 1 < len) d[e0 + 1] = (uint16_t)h1;
            if (e0 + 2 < len) d[e0 + 2] = (uint16_t)h2;
            if (e0 + 3 < len) d[e0 + 3] = (uint16_t)h3;
        }
    }
}

// 16-bit output of a full wave tile whose first element lies on the 16-byte
// grid, two chunks (2p and 2p + 1) at a time.  A lane's four words of a chunk
// make only 8 bytes, so neighbouring lanes trade halves (one DPP swap per
// dword): the even lane stores 16 bytes of chunk 2p, the odd lane 16 bytes of
// chunk 2p + 1.  The bytes written are those of store_unpacked per chunk.
__device__ __forceinline__ uint32_t swap_with_neighbour_lane(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF,
                                                 0xF, false);
}

template <int OUT>
__device__ __forceinline__ void store_half_chunk_pair(uint16_t *dst, int p, int lane,
                                                      const u32x4 ua, const u32x4 ub) {
    const bool odd = (lane & 1) != 0;
    const uint32_t a0 = to_half_bits<OUT>(ua.x) | (to_half_bits<OUT>(ua.y) << 16);
    const uint32_t a1 = to_half_bits<OUT>(ua.z) | (to_half_bits<OUT>(ua.w) << 16);
    const uint32_t b0 = to_half_bits<OUT>(ub.x) | (to_half_bits<OUT>(ub.y) << 16);
    const uint32_t b1 = to_half_bits<OUT>(ub.z) | (to_half_bits<OUT>(ub.w) << 16);
    const uint32_t g0 = swap_with_neighbour_lane(odd ? a0 : b0);
    const uint32_t g1 = swap_with_neighbour_lane(odd ? a1 : b1);
    u32x4 o;
    o.x = odd ? g0 : a0;
    o.y = odd ? g1 : a1;
    o.z = odd ? b0 : g0;
    o.w = odd ? b1 : g1;
    const int e0 = 4 * ((2 * p + (odd ? 1 : 0)) * kWave + (lane & ~1));
    store_streaming16(dst + e0, o);
}

// The unpacked words u[j] (chunk j) of a wave tile -> dst, in either format.
template <int OUT>
__device__ __forceinline__ void store_unpacked_tile(void *dst, int len, int lane,
                                                    const u32x4 (&u)[kChunksPerLane]) {
    if (OUT != kOutFp32 && len == kWaveTile && ((uintptr_t)dst & 15u) == 0) {   // wave uniform
#pragma unroll
        for (int p = 0; p < kChunksPerLane / 2; ++p)
            store_half_chunk_pair<OUT>((uint16_t *)dst, p, lane, u[2 * p], u[2 * p + 1]);
        return;
    }
    const bool dst_dw = ((uintptr_t)dst & 3u) == 0;        // wave uniform
#pragma unroll
    for (int j = 0; j < kChunksPerLane; ++j) {
        const int e0 = 4 * (j * kWave + lane);
        if (e0 < len) store_unpacked<OUT>(dst, e0, len, u[j], dst_dw);
    }
}

// ---------------------------------------------------------------------------
// Unpack one wave tile: len*R stream bytes at src -> `len` FP32 words at dst.
// [buf_lo, buf_hi) is the whole packed buffer: a 16-byte piece inside it may
// be read whole even where it reaches into a neighbouring tile.
// ---------------------------------------------------------------------------
template <int R, int OUT = kOutFp32>
__device__ __forceinline__ void unpack_wave_tile(const uint8_t *__restrict__ src,
                                                 void *__restrict__ dst, int len,
                                                 const uint8_t *buf_lo,
                                                 const uint8_t *buf_hi, uint32_t *lds,
                                                 int lane) {
    const uint32_t s = (uint32_t)((uintptr_t)src & 15u);   // wave uniform
    const bool full = (len == kWaveTile);

    if (full && s == 0) {
        constexpr int kPieces = R * kChunksPerLane / 4;     // 16-byte pieces per lane
        u32x4 v[kPieces];
#pragma unroll
        for (int k = 0; k < kPieces; ++k)
            v[k] = load_stream16(src + 16 * (k * kWave + lane));
#pragma unroll
        for (int k = 0; k < kPieces; ++k) *(u32x4 *)(lds + 4 * (k * kWave + lane)) = v[k];
        wave_lds_sync();
        u32x4 u[kChunksPerLane];
#pragma unroll
        for (int j = 0; j < kChunksPerLane; ++j) {
            const int c = j * kWave + lane;
            uint32_t y[4];
#pragma unroll
            for (int t = 0; t < R; ++t) y[t] = lds[c * R + t];
            u[j] = shift_to_top<R>(y);
        }
        store_unpacked_tile<OUT>(dst, len, lane, u);
        return;
    }

    const int nbytes = len * R;
    const uint8_t *src_al = src - s;
    const int npieces = (int)(s + nbytes + 15) >> 4;       // <= kWaveTile / 4 + 1
    for (int k = 0; k * kWave < npieces; ++k) {
        const int q = k * kWave + lane;
        if (q < npieces) {
            const uint8_t *a = src_al + 16 * q;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (a >= buf_lo && a + 16 <= buf_hi) {
                v = load_stream16(a);
            } else {
                uint32_t w[4] = {0u, 0u, 0u, 0u};
                for (int t = 0; t < 16; ++t)
                    if (a + t >= buf_lo && a + t < buf_hi)
                        w[t >> 2] |= (uint32_t)a[t] << (8 * (t & 3));
                v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
            }
            *(u32x4 *)(lds + 4 * q) = v;
        }
    }
    wave_lds_sync();

    // Stream byte b of the tile sits at LDS byte b + s.
    const uint32_t sh = s & 3u;
    u32x4 u[kChunksPerLane];
#pragma unroll
    for (int j = 0; j < kChunksPerLane; ++j) {
        const int c = j * kWave + lane;
        u[j] = u32x4{0u, 0u, 0u, 0u};
        if (4 * c < len) {
            const int d = (int)(s + 4 * c * R) >> 2;        // <= kWaveTile - 1
            uint32_t x[5];
#pragma unroll
            for (int t = 0; t <= R; ++t) x[t] = lds[d + t];
            uint32_t y[4];
#pragma unroll
            for (int t = 0; t < R; ++t) y[t] = funnel(x[t + 1], x[t], sh);
            u[j] = shift_to_top<R>(y);
        }
    }
    store_unpacked_tile<OUT>(dst, len, lane, u);
}

// ---------------------------------------------------------------------------
// Block -> (layer, tile) through the offset table, wave -> wave tile.
// ---------------------------------------------------------------------------
struct TileRef {
    int64_t elem;      // first weight of the wave tile (absolute index)
    int64_t byte;      // first stream byte of the wave tile
    int len;           // weights in the wave tile, 0 = nothing to do
    int r;
};

template <bool INLINE, int WAVES = kWavesPerBlock>
__device__ __forceinline__ TileRef locate(const PackArgs &a, uint32_t block, int wave) {
    const uint32_t *tile_off = INLINE ? a.inl.tile_off : a.dev.tile_off;
    const int64_t *elem_off = INLINE ? a.inl.elem_off : a.dev.elem_off;
    const int64_t *pack_off = INLINE ? a.inl.pack_off : a.dev.pack_off;
    const uint8_t *rbytes = INLINE ? a.inl.rbytes : a.dev.rbytes;
    int lo = 0, hi = a.n_layers;            // largest lo with tile_off[lo] <= block
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (table_load(tile_off, mid) <= block) lo = mid; else hi = mid;
    }
    const int64_t e_begin = table_load(elem_off, lo);
    const int64_t n = table_load(elem_off, lo + 1) - e_begin;
    const int64_t first = (int64_t)(block - table_load(tile_off, lo)) * (WAVES * kWaveTile) +
                          (int64_t)wave * kWaveTile;
    TileRef t;
    t.r = table_byte(rbytes, lo);
    t.elem = e_begin + first;
    t.byte = table_load(pack_off, lo) + first * t.r;
    const int64_t left = n - first;
    t.len = left <= 0 ? 0 : (left < kWaveTile ? (int)left : kWaveTile);
    return t;
}

}  // namespace adt
