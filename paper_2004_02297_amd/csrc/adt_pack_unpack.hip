// ADT Bitpack / Bitunpack for gfx950 (Section III, Algorithms 2 and 5 of
// arXiv 2004.02297), all layers in one launch.
//
// Work decomposition.  A wavefront owns a "wave tile" of 1024 consecutive
// weights of one layer.  A wave moves its tile in three steps and never talks
// to another wave, so there is no block barrier and a block may hold one
// wavefront (the default: see the launch shapes in adt_tables.h) or four:
//   pack   : 4 coalesced 128-bit loads per lane of FP32 words
//            -> keep the top r bytes of every word in registers
//            -> write the r-byte stream to the wave's LDS slice
//            -> read it back as 16-byte pieces in stream order
//            -> 128-bit stores on 16-byte aligned addresses of the stream.
//   unpack : the mirror image (aligned 128-bit loads of the stream -> LDS ->
//            r(+1) dwords per 4 weights -> shift each weight's bytes to the
//            top of a zeroed word -> 128-bit stores of FP32).
// The stream side is always accessed on the 16-byte grid of absolute
// addresses, whatever the layer's start offset is: a misaligned tile reads
// its LDS slice at a shifted position (funnel shift by the byte phase) and
// only the first and last piece of a tile fall back to byte accesses.
// The FP32 side needs 4-byte alignment only; the hardware splits a 128-bit
// access that is not 16-byte aligned.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_launch.h"
#include "adt_tables.h"
#include "adt_tile_ops.h"

namespace adt {

// ---------------------------------------------------------------------------
// Kernels: block -> (layer, tile) through the offset table, wave -> wave tile.
// ---------------------------------------------------------------------------
template <bool INLINE, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void pack_kernel(const PackArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[WAVES][kWaveLdsDw];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const TileRef t = locate<INLINE, WAVES>(a, blockIdx.x, wave);
    if (t.len == 0) return;
    const uint32_t *src = a.weights + t.elem;
    uint8_t *dst = a.packed + t.byte;
    uint32_t *lds = smem[wave];
    const bool nt = a.packed_size > a.stream_cache_limit;
    switch (t.r) {
        case 1: pack_wave_tile<1>(src, dst, t.len, lds, lane, nt); break;
        case 2: pack_wave_tile<2>(src, dst, t.len, lds, lane, nt); break;
        case 3: pack_wave_tile<3>(src, dst, t.len, lds, lane, nt); break;
        default: pack_wave_tile<4>(src, dst, t.len, lds, lane, nt); break;
    }
}

template <bool INLINE, int OUT>
__global__ __launch_bounds__(kUnpackWaves * kWave) void unpack_kernel(const PackArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t smem[kUnpackWaves][kWaveLdsDw];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const TileRef t = locate<INLINE, kUnpackWaves>(a, blockIdx.x, wave);
    if (t.len == 0) return;
    const uint8_t *src = a.packed + t.byte;
    // a.weights is the output buffer here: FP32 words or 16-bit elements
    void *dst = OUT == kOutFp32
                    ? (void *)(const_cast<uint32_t *>(a.weights) + t.elem)
                    : (void *)((uint16_t *)const_cast<uint32_t *>(a.weights) + t.elem);
    const uint8_t *lo = a.packed;
    const uint8_t *hi = a.packed + a.packed_size;
    uint32_t *lds = smem[wave];
    switch (t.r) {
        case 1: unpack_wave_tile<1, OUT>(src, dst, t.len, lo, hi, lds, lane); break;
        case 2: unpack_wave_tile<2, OUT>(src, dst, t.len, lo, hi, lds, lane); break;
        case 3: unpack_wave_tile<3, OUT>(src, dst, t.len, lo, hi, lds, lane); break;
        default: unpack_wave_tile<4, OUT>(src, dst, t.len, lo, hi, lds, lane); break;
    }
}

// waves: 1 or 4 (the tile table must have been built for waves * 1024 weights per block)
hipError_t launch_pack(const PackArgs &a, uint32_t n_tiles, bool inline_table, int waves,
                       uint32_t extra_lds, hipStream_t stream) {
    void (*k)(PackArgs);
    if (waves == 1) k = inline_table ? pack_kernel<true, 1> : pack_kernel<false, 1>;
    else k = inline_table ? pack_kernel<true, 4> : pack_kernel<false, 4>;
    return launch(k, kKernelPack, n_tiles, waves * kWave, stream, a, extra_lds);
}

hipError_t launch_unpack(const PackArgs &a, uint32_t n_tiles, bool inline_table, int out_format,
                         uint32_t extra_lds, hipStream_t stream) {
    void (*k)(PackArgs);
    if (inline_table)
        k = out_format == kOutFp32   ? unpack_kernel<true, kOutFp32>
            : out_format == kOutBf16 ? unpack_kernel<true, kOutBf16>
                                     : unpack_kernel<true, kOutFp16>;
    else
        k = out_format == kOutFp32   ? unpack_kernel<false, kOutFp32>
            : out_format == kOutBf16 ? unpack_kernel<false, kOutBf16>
                                     : unpack_kernel<false, kOutFp16>;
    return launch(k, out_format == kOutFp32 ? kKernelUnpack : kKernelUnpack16, n_tiles,
                  kUnpackWaves * kWave, stream, a, extra_lds);
}

}  // namespace adt
