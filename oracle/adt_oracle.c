/*
 * CPU oracle for Approximate Data Transfer (ADT) and Adaptive Weight Precision
 * (AWP), arXiv 2004.02297.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is a plain, slow,
 * single-threaded, scalar reference written from the paper's definitions, used
 * only to check the GPU library and to be timed beside it as a CPU baseline.
 * It shares no code, header, table or helper with the GPU implementation.
 *
 * Pins (see tests/test_oracle_*.py): closed-form mask over all 2^32 bit
 * patterns, hand-derived IEEE-754 worked examples, bfloat16 widening, memcpy at
 * 4 bytes, an independent numpy byte-slicing formulation, numpy/torch norms,
 * hand-computed AWP trajectories.  The only part no source outside this
 * repository fixes is the ORDER of the kept bytes inside one packed element
 * (the paper leaves it open); it is fixed by the library header: little endian.
 *
 * Build: gcc -O2 -shared -fPIC -o liboracle.so adt_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* Number of per-layer statistics and their order: sum of squares, l2-norm,
 * largest magnitude. */
#define ORACLE_NSTATS 3

/*
 * Bitpack (Section III-A, Algorithm 2; truncation rule of Section III: a weight
 * is a 32-bit word and keeping N bits drops its 32-N lowest bits).
 *
 * For every layer, walk its weights in order; copy the RoundTo most
 * significant bytes of each weight to Pw and advance the running byte offset
 * by RoundTo.  The offset keeps running across layers, so the layers' streams
 * are concatenated without padding.  The kept bytes of one weight are stored
 * low-order byte first (the order they have in a little-endian FP32 image).
 *
 * Returns the total number of bytes written, or -1 on an invalid table.
 */
int64_t oracle_pack(const float *W, const int64_t *layer_offsets,
                    const uint8_t *bytes_per_layer, int n_layers, uint8_t *Pw)
{
    int64_t POffset = 0;
    for (int layer = 0; layer < n_layers; ++layer) {
        int RoundTo = bytes_per_layer[layer];
        if (RoundTo < 1 || RoundTo > 4) return -1;
        if (layer_offsets[layer + 1] < layer_offsets[layer]) return -1;
        for (int64_t i = layer_offsets[layer]; i < layer_offsets[layer + 1]; ++i) {
            uint32_t word;
            memcpy(&word, &W[i], 4);            /* the weight as a 32-bit word */
            int dropped = 4 - RoundTo;          /* low-order bytes discarded   */
            for (int k = 0; k < RoundTo; ++k) {
                /* byte number (dropped + k) of the word, counting from the
                 * least significant byte */
                Pw[POffset + k] = (uint8_t)((word >> (8 * (dropped + k))) & 0xFFu);
            }
            POffset += RoundTo;
        }
    }
    return POffset;
}

/*
 * Bitunpack (Section III-C, Algorithm 5): each weight is the RoundTo-byte
 * integer found at the running offset, shifted left by (4 - RoundTo) * 8 bits;
 * the bits that come back in are zero.
 *
 * Returns the total number of bytes consumed, or -1 on an invalid table.
 */
int64_t oracle_unpack(const uint8_t *Pw, const int64_t *layer_offsets,
                      const uint8_t *bytes_per_layer, int n_layers, float *W)
{
    int64_t POffset = 0;
    for (int layer = 0; layer < n_layers; ++layer) {
        int RoundTo = bytes_per_layer[layer];
        if (RoundTo < 1 || RoundTo > 4) return -1;
        if (layer_offsets[layer + 1] < layer_offsets[layer]) return -1;
        for (int64_t i = layer_offsets[layer]; i < layer_offsets[layer + 1]; ++i) {
            uint32_t q = 0;
            for (int k = 0; k < RoundTo; ++k)
                q |= (uint32_t)Pw[POffset + k] << (8 * k);
            uint32_t word = q << ((4 - RoundTo) * 8);
            memcpy(&W[i], &word, 4);
            POffset += RoundTo;
        }
    }
    return POffset;
}

/*
 * Per-layer statistics used by AWP (Section II: the l2-norm of all weights of
 * a layer, computed every batch on the full-precision master weights).
 *
 * stats[layer][0] = sum over the layer of w^2, accumulated in double precision
 *                   in index order,
 * stats[layer][1] = sqrt of that sum (the l2-norm |W_layer|),
 * stats[layer][2] = largest |w| of the layer (NaN if any weight is NaN).
 * An empty layer gives 0, 0, 0.
 */
void oracle_stats(const float *W, const int64_t *layer_offsets, int n_layers,
                  double *stats)
{
    for (int layer = 0; layer < n_layers; ++layer) {
        double sumsq = 0.0;
        double absmax = 0.0;
        int saw_nan = 0;
        for (int64_t i = layer_offsets[layer]; i < layer_offsets[layer + 1]; ++i) {
            double w = (double)W[i];
            sumsq += w * w;
            if (isnan(w)) saw_nan = 1;
            else if (fabs(w) > absmax) absmax = fabs(w);
        }
        stats[layer * ORACLE_NSTATS + 0] = sumsq;
        stats[layer * ORACLE_NSTATS + 1] = sqrt(sumsq);
        stats[layer * ORACLE_NSTATS + 2] = saw_nan ? (double)NAN : absmax;
    }
}

/*
 * Norms of layer groups (Section IV-B: for ResNet the precision is adapted per
 * building block, not per layer).  Group g is the run of layers
 * [group_offsets[g], group_offsets[g+1]); its norm is the l2-norm of all
 * weights of those layers, squares accumulated in double in index order.
 */
void oracle_group_norms(const float *W, const int64_t *layer_offsets,
                        const int32_t *group_offsets, int n_groups, double *l2_group)
{
    for (int g = 0; g < n_groups; ++g) {
        double sumsq = 0.0;
        int64_t first = layer_offsets[group_offsets[g]];
        int64_t last = layer_offsets[group_offsets[g + 1]];
        for (int64_t i = first; i < last; ++i) {
            double w = (double)W[i];
            sumsq += w * w;
        }
        l2_group[g] = sqrt(sumsq);
    }
}

/*
 * One batch of the AWP rule for all layers (Section II, Algorithm 1).
 *
 * Per layer: delta = (|W_b| - |W_{b-1}|) / |W_{b-1}|; when delta < T the
 * layer's interval counter goes up by one; when the counter equals INTERVAL
 * the layer gains N bits and the counter returns to zero.  The counter is
 * cumulative: a batch with delta >= T leaves it unchanged (the algorithm has
 * no else-branch).  The number of bytes sent for a layer is its bit count
 * rounded up to whole bytes (Section III-A: 14 bits -> 2 bytes).
 *
 * Readings where the paper is silent: the first batch has no predecessor and
 * only records the norm; bits are capped at 32; a zero previous norm gives
 * delta = 0 when the norm is still zero and +infinity otherwise.
 */
void oracle_awp_update(const double *l2_now, double *l2_prev, int32_t *counter,
                       int32_t *bits, uint8_t *bytes_out, int n_layers,
                       double T, int INTERVAL, int N, int is_first_batch)
{
    for (int layer = 0; layer < n_layers; ++layer) {
        if (!is_first_batch) {
            double delta;
            if (l2_prev[layer] == 0.0)
                delta = (l2_now[layer] == 0.0) ? 0.0 : (double)INFINITY;
            else
                delta = (l2_now[layer] - l2_prev[layer]) / l2_prev[layer];
            if (delta < T)
                counter[layer] += 1;
            if (counter[layer] == INTERVAL) {
                bits[layer] += N;
                if (bits[layer] > 32) bits[layer] = 32;
                counter[layer] = 0;
            }
        }
        l2_prev[layer] = l2_now[layer];
        bytes_out[layer] = (uint8_t)((bits[layer] + 7) / 8);
    }
}
