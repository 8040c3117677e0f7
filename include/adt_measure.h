/*
 * libadt measurement aids: exact per-launch kernel durations and ablation
 * variants of the pack / unpack kernels.  Nothing here is needed to use the
 * method; a benchmark includes this header next to adt.h.  Same conventions
 * as adt.h (C ABI, negative adt_status on error).
 */
#ifndef ADT_MEASURE_H_
#define ADT_MEASURE_H_

#include "adt.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch timing (measurement aid, off by default).  While enabled, every
 * kernel the library launches carries the dispatch's own begin / end
 * timestamps (this costs the host about 10 us per launch, so a benchmark
 * switches it on for a sample of its steps).  adt_timing_enable(on, n) also
 * prepares event pairs for n launches ahead of time.  adt_timing_read waits
 * for the launches recorded so far, writes per-kernel totals to `out` (host,
 * ADT_NKERNELS entries, indexed as adt_kernel_name names them) and forgets
 * them.
 */
#define ADT_NKERNELS 10
typedef struct adt_kernel_time {
    int64_t launches;
    double total_ms;
    double min_ms;
    double max_ms;
} adt_kernel_time;
int adt_timing_enable(int on, int reserve_launches);
int adt_timing_read(adt_kernel_time *out);
const char *adt_kernel_name(int kernel);   /* "" outside 0..ADT_NKERNELS-1 */

/*
 * Launch shape of a streaming kernel (tuning aid): wavefronts per block and a
 * number of bytes of dynamic LDS that the kernel never touches, which lowers
 * the number of blocks a compute unit holds at once.  kernel: the index of
 * "pack_kernel", "unpack_kernel", "pack_unpack_kernel", "fused_kernel" or
 * "stats_partial_kernel" (adt_kernel_name); waves: 1 or 4 (unpack_kernel: 1,
 * stats_partial_kernel: 4), or 0 to return to the library's own choice.
 * Results do not depend on the shape, bit for bit.
 */
int adt_launch_shape(int kernel, int waves, int extra_lds_bytes);

/*
 * Size limit of the cache-friendly stream stores (tuning aid).  A kernel writes
 * a packed stream of at most this many bytes with ordinary stores, so that a
 * consumer right behind it can find the stream in the last-level cache, and a
 * larger one with nontemporal stores.  kernel: the index of "pack_kernel" (its
 * own limit, 320 MiB by default: adt_unpack usually follows), or of
 * "pack_unpack_kernel" / "fused_kernel" (one shared limit, 0 by default: always
 * nontemporal).  bytes >= 0 sets the limit for later calls (INT64_MAX: never
 * nontemporal) and returns the previous value; bytes < 0 only returns the
 * current value; negative adt_status for another kernel.  The stream's bytes
 * are the same either way.
 */
int64_t adt_stream_cache_limit(int kernel, int64_t bytes);

/*
 * Ablation variants of adt_pack / adt_unpack (same arguments, same bytes; for
 * measurement of the design choices only, not for production use):
 *   ADT_ABLATION_NAIVE       one thread per weight, byte accesses on the stream
 *                            (the per-weight loops of Algorithms 2 and 5 as
 *                            written), all layers in one launch
 *   ADT_ABLATION_VEC_DIRECT  128-bit loads, register byte selection, one
 *                            4r-byte store per lane, no LDS pass (pack only;
 *                            layer starts must be 4-byte aligned)
 *   ADT_ABLATION_PER_LAYER   the production kernel, one launch per layer
 * `unpack` != 0 runs the unpack direction (then `weights` is written).
 * NAIVE and VEC_DIRECT take at most 128 layers.
 */
#define ADT_ABLATION_NAIVE 1
#define ADT_ABLATION_VEC_DIRECT 2
#define ADT_ABLATION_PER_LAYER 3
int adt_ablation(int variant, int unpack, const float *weights, const int64_t *layer_offsets,
                 const uint8_t *bytes_per_layer, int n_layers, uint8_t *packed,
                 adt_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* ADT_MEASURE_H_ */
