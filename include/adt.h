/*
 * libadt — Approximate Data Transfer (ADT) pack / unpack and the Adaptive
 * Weight Precision (AWP) per-layer statistics of arXiv 2004.02297, for AMD
 * MI355X (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * Conventions common to all calls
 *   - "device" pointers are HIP device memory of the CURRENT device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer.
 *   - The small per-layer tables (layer_offsets, bytes_per_layer) are HOST
 *     arrays.  They are read during the call and may be changed or freed as
 *     soon as it returns.
 *   - layer_offsets has n_layers + 1 entries in ELEMENT units:
 *     layer_offsets[0] == 0, non-decreasing, layer_offsets[n_layers] == N.
 *     All layers' weights are contiguous in one FP32 buffer.  Empty layers
 *     are legal.
 *   - bytes_per_layer[l] in {1, 2, 3, 4} is the layer's "RoundTo".
 *   - GPU work is enqueued on `stream` (a hipStream_t; NULL is the default
 *     stream) and the call returns without waiting for it.
 *   - Return value: ADT_OK (0) or a negative adt_status.  Arguments are
 *     validated before anything is launched; on error nothing is written.
 *     n_layers == 0 or N == 0 succeeds without a launch.
 *   - No call throws or exits.  adt_strerror() gives a text for a status and
 *     adt_last_error() the detail of the calling thread's last failure.
 *
 * Packed stream (wire format written by adt_pack, read by adt_unpack)
 *   Layer l starts at byte P_l = sum_{j<l} n_j * r_j: the running byte offset
 *   of Bitpack (Algorithm 2) carried across layers, no padding anywhere.
 *   Weight i of layer l occupies bytes [P_l + i*r_l, P_l + (i+1)*r_l) and
 *   holds the r_l most significant bytes of its 32-bit IEEE-754 word
 *   (Section III: keeping N bits discards the 32-N lowest bits), least
 *   significant kept byte first.  With r = 4 the stream is a copy of the
 *   weights; with r = 2 it is an array of bfloat16 obtained by truncation.
 *   The paper does not fix the byte order inside an element; this header does.
 */
#ifndef ADT_H_
#define ADT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *adt_stream_t;

enum adt_status {
    ADT_OK = 0,
    ADT_EINVAL = -1,  /* null pointer, n_layers < 0, byte count outside 1..4,
                         offsets not starting at 0 or decreasing              */
    ADT_EALIGN = -2,  /* a float buffer is not 4-byte aligned                  */
    ADT_EHIP = -3,    /* HIP runtime / launch failure (see adt_last_error)     */
    ADT_ENOMEM = -4,  /* the library's scratch memory could not be allocated   */
    ADT_ERANGE = -5   /* sizes exceed what one launch can address              */
};

/* Number of statistics awp_layer_stats writes per layer, and their order. */
#define AWP_NSTATS 3
#define AWP_STAT_SUMSQ 0   /* sum of w^2                     */
#define AWP_STAT_L2 1      /* sqrt of it: the l2-norm |W_l|  */
#define AWP_STAT_ABSMAX 2  /* largest |w|                    */

/*
 * Size in bytes of the packed stream: sum over layers of n_l * r_l
 * (Algorithm 2's final POffset).  Host only, no GPU.  Negative adt_status on
 * an invalid table.
 */
int64_t adt_packed_size(const int64_t *layer_offsets /* host */,
                        const uint8_t *bytes_per_layer /* host */,
                        int n_layers);

/*
 * Bitpack (Section III-A, Algorithm 2) of all layers in one launch.
 *   weights  device, N floats, 4-byte aligned (16-byte alignment is fastest)
 *   out      device, at least adt_packed_size(...) bytes, any alignment; must
 *            not overlap `weights`.  Bytes beyond the packed size are not
 *            touched.
 */
int adt_pack(const float *weights, const int64_t *layer_offsets,
             const uint8_t *bytes_per_layer, int n_layers, uint8_t *out,
             adt_stream_t stream);

/*
 * Bitunpack (Section III-C, Algorithm 5) of all layers in one launch: every
 * weight becomes its r stored bytes shifted left by 8*(4-r) bits, the low
 * bits zero.  Hence unpack(pack(w)) == bits(w) & (0xFFFFFFFF << 8*(4-r)).
 *   packed       device, stream written by adt_pack with the same two tables
 *   weights_out  device, N floats, 4-byte aligned; must not overlap `packed`
 */
int adt_unpack(const uint8_t *packed, const int64_t *layer_offsets,
               const uint8_t *bytes_per_layer, int n_layers,
               float *weights_out, adt_stream_t stream);

/*
 * Bitunpack straight to a 16-bit compute format (the paper's related-work
 * section proposes decompressing to half precision to combine the method with
 * mixed-precision training).  Same stream and tables as adt_unpack; element i
 * of `out` is made from the FP32 word w'_i that adt_unpack would return:
 *   ADT_OUT_BF16  the top 16 bits of w'_i (truncation, as ADT itself truncates;
 *                 exact for r <= 2)
 *   ADT_OUT_FP16  w'_i converted to IEEE binary16, round to nearest even,
 *                 overflow to infinity; a NaN becomes the quiet NaN 0x7E00 with
 *                 the sign of w'_i, whatever its payload
 *   out  device, N 16-bit elements, 2-byte aligned (4-byte alignment of every
 *        layer start is the fast case); must not overlap `packed`
 */
#define ADT_OUT_BF16 1
#define ADT_OUT_FP16 2
int adt_unpack16(const uint8_t *packed, const int64_t *layer_offsets,
                 const uint8_t *bytes_per_layer, int n_layers, uint16_t *out, int format,
                 adt_stream_t stream);

/*
 * adt_pack and adt_unpack of the same weights in one kernel: the weights are
 * read once; `out` receives the packed stream exactly as adt_pack writes it
 * and `weights_out` the FP32 words adt_unpack would return from that stream
 * (bits(w) & (0xFFFFFFFF << 8*(4-r))).  For the device that packs for its
 * peers and also needs the truncated weights itself.
 *   weights_out  device, N floats, 4-byte aligned; must not overlap the others
 */
int adt_pack_unpack(const float *weights, const int64_t *layer_offsets,
                    const uint8_t *bytes_per_layer, int n_layers, uint8_t *out,
                    float *weights_out, adt_stream_t stream);

/*
 * Per-layer statistics AWP monitors (Section II: the l2-norm of all weights
 * of a layer, every batch, on the full-precision weights).
 *   stats_out  device, n_layers * AWP_NSTATS doubles, row l =
 *              { sum w^2, sqrt(sum w^2), max |w| }.  Squares and sums are
 *              taken in double precision; partial sums are combined in a
 *              fixed order, so results are identical from run to run.  An
 *              empty layer gives {0, 0, 0}; a NaN weight makes all three NaN.
 * Uses per-device scratch memory owned by the library (grown on demand, kept
 * until adt_shutdown).  Calls on different streams of one device are ordered
 * against each other by the library (a call waits, on the GPU, for the previous
 * call's kernels before it reuses the scratch); calls from different host
 * threads are serialised by a lock.
 * The plan path (awp_adt_step) adds the same exact squares over tiles of 4096
 * weights instead of 8192, so the two paths' sums agree to rounding (about
 * 1e-15 relative), not bit for bit: an AWP decision whose delta lies within
 * that distance of T may differ between them.
 */
int awp_layer_stats(const float *weights, const int64_t *layer_offsets,
                    int n_layers, double *stats_out, adt_stream_t stream);

/*
 * awp_layer_stats for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bit-identical results as awp_layer_stats,
 * but the partial sums live in a fixed array inside the library's device image
 * (AWP_NOALLOC_MAX_TILES * 12 bytes = 1.5 MiB, held by every GPU the library
 * runs on until the process ends) and the call never allocates or frees
 * anything, on the host side of HIP or on the device.
 * Limits (ADT_ERANGE beyond them, nothing launched): n_layers <= 128, and
 * sum over layers of ceil(n_l / 8192) <= AWP_NOALLOC_MAX_TILES (about 1.07 G
 * weights).
 * All calls on one GPU share that array: calls that overlap in time on one GPU
 * (different streams without ordering, or different host threads) race and
 * give wrong statistics; order them on one stream or with events.  The array
 * keeps the last call's partials; nothing in it needs clearing between calls.
 * The first call on a device looks up the array's device address; make that
 * call outside a graph capture.
 */
#define AWP_NOALLOC_MAX_TILES 131072
int awp_layer_stats_noalloc(const float *weights, const int64_t *layer_offsets,
                            int n_layers, double *stats_out, adt_stream_t stream);

/*
 * One batch of the AWP rule (Section II, Algorithm 1) for all layers.  Host
 * only, no GPU; all pointers are host arrays of n_layers entries.
 *   delta = (l2_now - l2_prev) / l2_prev; if delta < T the layer's counter
 *   goes up by one; if the counter equals `interval` the layer gains `n_bits`
 *   bits (capped at 32) and its counter returns to zero.  The counter is
 *   cumulative (Algorithm 1 has no else-branch).  Then l2_prev := l2_now and
 *   bytes_out[l] = ceil(bits[l] / 8) (Section III-A: 14 bits -> 2 bytes).
 *   With is_first_batch != 0 only l2_prev and bytes_out are written.  A zero
 *   previous norm gives delta = 0 if the norm is still zero, else +infinity.
 */
int awp_update(const double *l2_now, double *l2_prev, int32_t *counter,
               int32_t *bits, uint8_t *bytes_out, int n_layers, double T,
               int interval, int n_bits, int is_first_batch);

/*
 * Plan: the whole pass with device-resident AWP state, asynchronous.
 *
 * A plan owns, on the current device, the per-layer tables, the AWP state
 * (bits, interval counters, previous norms) and scratch for the statistics.
 * awp_adt_step enqueues on `stream`, without waiting for the GPU, exactly what
 *     awp_layer_stats(weights) -> awp_update(state) -> adt_pack(weights,
 *     bytes) -> adt_unpack(packed, bytes) into weights_out
 * computes in that order (Algorithm 1's order: the byte counts chosen from this
 * batch's norms are the ones this batch is packed with), but reads the weights
 * from HBM once: statistics, stream and truncated weights are produced by one
 * kernel under the assumption that the byte counts of the previous batch still
 * hold, the rule then runs on the device, and only if it changed a byte count
 * (a few times per training run) are stream and truncated weights redone.
 *   layer_offsets  host, as for adt_pack
 *   init_bits      host, n_layers entries, or NULL for 8 bits everywhere
 *                  (Section V-A: AWP starts at 8 bits)
 *   T, interval, n_bits  parameters of Algorithm 1
 *   weights        device, N floats, 4-byte aligned
 *   packed         device, packed_capacity bytes; capacity must be at least
 *                  4*N so that any byte assignment fits
 *   weights_out    device, N floats, or NULL to skip the truncated copy; must
 *                  not overlap weights or packed
 * Calls on one plan must be issued from one thread at a time and on one stream
 * (or on streams ordered by the caller).  The step allocates nothing and does
 * not wait for the GPU, so it may be captured into a HIP graph and replayed:
 * all state that changes from batch to batch lives on the device.  (An eager
 * step leaves the redo launch out while the host can tell, from a status word
 * the device publishes, that no interval counter can reach INTERVAL in this
 * batch; a captured step always contains it.)
 * awp_plan_read waits for the steps enqueued so far and copies the state to
 * host arrays (any pointer may be NULL): stats n_layers*AWP_NSTATS doubles,
 * bits / counter / bytes n_layers entries, packed_size one value.
 */
typedef struct awp_plan awp_plan;
int awp_plan_create(const int64_t *layer_offsets, int n_layers, const int32_t *init_bits,
                    double T, int interval, int n_bits, awp_plan **plan_out);
int awp_adt_step(awp_plan *plan, const float *weights, uint8_t *packed,
                 int64_t packed_capacity, float *weights_out, adt_stream_t stream);
/* awp_adt_step with the truncated weights written in a 16-bit format (see
 * adt_unpack16): weights_out holds N 16-bit elements, 2-byte aligned. */
int awp_adt_step16(awp_plan *plan, const float *weights, uint8_t *packed,
                   int64_t packed_capacity, uint16_t *weights_out, int format,
                   adt_stream_t stream);
int awp_plan_read(awp_plan *plan, double *stats, int32_t *bits, int32_t *counter,
                  uint8_t *bytes, int64_t *packed_size);
/*
 * While no byte count can move (see above), an eager step leaves the final
 * reduction of its statistics and the rule to the next step, whose first kernel
 * carries them along; the packed stream and the truncated weights are complete
 * in stream order all the same.  awp_plan_flush enqueues that leftover work now,
 * on the stream of the last step, without waiting (no-op if there is none), for
 * a caller that wants the plan's state settled in stream order, e.g. before an
 * event.  awp_plan_read, awp_plan_get_state and awp_plan_set_state do the same
 * by themselves.  Capturing a step while such work is left over is refused with
 * ADT_EINVAL: call one of these first.
 */
int awp_plan_flush(awp_plan *plan);
/*
 * Checkpoint / resume of a plan's AWP state (host arrays, one entry per layer,
 * or per group for a grouped plan; any pointer may be NULL).  get waits for
 * the steps enqueued so far; set replaces the state, recomputes the byte counts
 * and stream offsets from `bits`, and takes effect for the next step.
 *   l2_prev        the norms recorded by the last batch
 *   batches_seen   0 if no batch has been processed yet (the next batch then
 *                  only records norms), non-zero otherwise
 */
int awp_plan_get_state(awp_plan *plan, int32_t *bits, int32_t *counter, double *l2_prev,
                       int32_t *batches_seen);
int awp_plan_set_state(awp_plan *plan, const int32_t *bits, const int32_t *counter,
                       const double *l2_prev, int32_t batches_seen);
int awp_plan_destroy(awp_plan *plan);

/*
 * Layer groups.  Section IV-B: for ResNet the paper adapts the precision per
 * building block instead of per layer.  A group is a run of consecutive layers
 * [group_offsets[g], group_offsets[g+1]) (host array, n_groups + 1 entries,
 * group_offsets[0] == 0, non-decreasing, last entry == n_layers) that shares
 * one norm, the l2-norm over all weights of its layers, one AWP state and one
 * byte count.
 *   awp_group_norms         host only: l2_group[g] = sqrt(sum over the group's
 *                           layers of stats[l][AWP_STAT_SUMSQ]), layers added
 *                           in index order; feed it to awp_update with
 *                           n_groups in place of n_layers
 *   awp_expand_group_bytes  host only: bytes_layer[l] = bytes_group[g(l)]
 *   awp_plan_create_grouped as awp_plan_create with groups; init_bits has
 *                           n_groups entries (or NULL), and awp_plan_read
 *                           returns n_groups entries of bits / counter while
 *                           stats and bytes stay per layer
 */
int awp_group_norms(const double *stats, const int32_t *group_offsets, int n_groups,
                    double *l2_group);
int awp_expand_group_bytes(const uint8_t *bytes_group, const int32_t *group_offsets,
                           int n_groups, uint8_t *bytes_layer);
int awp_plan_create_grouped(const int64_t *layer_offsets, int n_layers,
                            const int32_t *group_offsets, int n_groups,
                            const int32_t *init_bits, double T, int interval, int n_bits,
                            awp_plan **plan_out);

/* Text for a status code (static string). */
const char *adt_strerror(int status);

/* Detail of the calling thread's most recent failure ("" if none). */
const char *adt_last_error(void);

/*
 * Digest of the source files this library was compiled from ("" if the build
 * did not record one).  A loader that has the sources compares it with their
 * digest to detect a library left over from older sources.
 */
const char *adt_source_digest(void);

/* Frees the library's per-device scratch memory.  Optional. */
int adt_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* ADT_H_ */
