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

/* A weight as its 32-bit IEEE-754 word, and back. */
static uint32_t word_of(float weight)
{
    uint32_t word;
    memcpy(&word, &weight, 4);
    return word;
}

static float weight_of(uint32_t word)
{
    float weight;
    memcpy(&weight, &word, 4);
    return weight;
}

/* Byte number `index` of a word, counting from the least significant byte. */
static uint8_t byte_of(uint32_t word, int index)
{
    return (uint8_t)((word >> (8 * index)) & 0xFFu);
}

/* 1 if the two tables describe layers this oracle can walk, else 0. */
static int tables_are_valid(const int64_t *layer_offsets, const uint8_t *bytes_per_layer,
                            int n_layers)
{
    for (int layer = 0; layer < n_layers; ++layer) {
        if (bytes_per_layer[layer] < 1 || bytes_per_layer[layer] > 4) return 0;
        if (layer_offsets[layer + 1] < layer_offsets[layer]) return 0;
    }
    return 1;
}

/*
 * Bitpack (Section III-A, Algorithm 2; truncation rule of Section III: a weight
 * is a 32-bit word and keeping N bits drops its 32-N lowest bits).
 *
 * A layer that keeps `keep` bytes per weight turns weight number i into the
 * `keep` most significant bytes of its word, at stream position
 * (start of the layer) + i * keep.  The layers' streams follow one another with
 * no padding, so a layer starts where the previous one ended.  The kept bytes
 * of one weight are stored low-order byte first (the order they have in a
 * little-endian FP32 image).
 *
 * Returns the total number of bytes written, or -1 on an invalid table.
 */
int64_t oracle_pack(const float *weights, const int64_t *layer_offsets,
                    const uint8_t *bytes_per_layer, int n_layers, uint8_t *stream)
{
    if (!tables_are_valid(layer_offsets, bytes_per_layer, n_layers)) return -1;
    int64_t layer_start = 0;                       /* stream byte where this layer begins */
    for (int layer = 0; layer < n_layers; ++layer) {
        const int keep = bytes_per_layer[layer];
        const int dropped = 4 - keep;              /* low-order bytes that are discarded */
        const float *layer_weights = weights + layer_offsets[layer];
        const int64_t count = layer_offsets[layer + 1] - layer_offsets[layer];
        for (int64_t i = 0; i < count; ++i) {
            const uint32_t word = word_of(layer_weights[i]);
            uint8_t *slot = stream + layer_start + i * keep;
            for (int b = 0; b < keep; ++b)
                slot[b] = byte_of(word, dropped + b);
        }
        layer_start += count * keep;
    }
    return layer_start;
}

/*
 * Bitunpack (Section III-C, Algorithm 5): a weight comes back as the integer
 * formed by its `keep` stored bytes, moved up by (4 - keep) * 8 bits; the bits
 * that come back in at the bottom are zero.
 *
 * Returns the total number of bytes consumed, or -1 on an invalid table.
 */
int64_t oracle_unpack(const uint8_t *stream, const int64_t *layer_offsets,
                      const uint8_t *bytes_per_layer, int n_layers, float *weights)
{
    if (!tables_are_valid(layer_offsets, bytes_per_layer, n_layers)) return -1;
    int64_t layer_start = 0;
    for (int layer = 0; layer < n_layers; ++layer) {
        const int keep = bytes_per_layer[layer];
        float *layer_weights = weights + layer_offsets[layer];
        const int64_t count = layer_offsets[layer + 1] - layer_offsets[layer];
        for (int64_t i = 0; i < count; ++i) {
            const uint8_t *slot = stream + layer_start + i * keep;
            uint32_t stored = 0;                   /* the kept bytes as one integer */
            for (int b = 0; b < keep; ++b)
                stored |= (uint32_t)slot[b] << (8 * b);
            layer_weights[i] = weight_of(stored << ((4 - keep) * 8));
        }
        layer_start += count * keep;
    }
    return layer_start;
}

/* Sum of the squares of weights [first, last), each square and the sum taken in
 * double precision, in index order. */
static double sum_of_squares(const float *weights, int64_t first, int64_t last)
{
    double total = 0.0;
    for (int64_t i = first; i < last; ++i) {
        const double w = (double)weights[i];
        total += w * w;
    }
    return total;
}

/*
 * Per-layer statistics used by AWP (Section II: the l2-norm of all weights of
 * a layer, computed every batch on the full-precision master weights).
 *
 * stats[layer][0] = sum over the layer of w^2 (double precision, index order),
 * stats[layer][1] = sqrt of that sum (the l2-norm |W_layer|),
 * stats[layer][2] = largest |w| of the layer (NaN if any weight is NaN).
 * An empty layer gives 0, 0, 0.
 */
void oracle_stats(const float *weights, const int64_t *layer_offsets, int n_layers,
                  double *stats)
{
    for (int layer = 0; layer < n_layers; ++layer) {
        const int64_t first = layer_offsets[layer], last = layer_offsets[layer + 1];
        double largest = 0.0;
        int has_nan = 0;
        for (int64_t i = first; i < last; ++i) {
            const double magnitude = fabs((double)weights[i]);
            if (isnan(magnitude)) has_nan = 1;
            else if (magnitude > largest) largest = magnitude;
        }
        const double squares = sum_of_squares(weights, first, last);
        double *row = stats + (size_t)layer * ORACLE_NSTATS;
        row[0] = squares;
        row[1] = sqrt(squares);
        row[2] = has_nan ? (double)NAN : largest;
    }
}

/*
 * Norms of layer groups (Section IV-B: for ResNet the precision is adapted per
 * building block, not per layer).  Group g is the run of layers
 * [group_offsets[g], group_offsets[g+1]); its norm is the l2-norm of all
 * weights of those layers (they are contiguous), squares added in index order.
 */
void oracle_group_norms(const float *weights, const int64_t *layer_offsets,
                        const int32_t *group_offsets, int n_groups, double *l2_group)
{
    for (int g = 0; g < n_groups; ++g) {
        const int64_t first = layer_offsets[group_offsets[g]];
        const int64_t last = layer_offsets[group_offsets[g + 1]];
        l2_group[g] = sqrt(sum_of_squares(weights, first, last));
    }
}

/* What AWP remembers about one layer from batch to batch. */
struct awp_layer_state {
    double previous_norm;
    int32_t counted;       /* batches counted towards the next precision step */
    int32_t bits;
};

/*
 * The rule of Section II / Algorithm 1 for one layer and one batch.  The
 * relative change of the norm against the previous batch is compared with the
 * threshold; a batch whose change lies below it is counted; when `interval`
 * batches have been counted the layer gains `step_bits` bits and the count
 * starts again.  A batch that is not counted leaves the count as it is (the
 * algorithm has no else-branch).  Readings where the paper is silent: bits stop
 * at 32; a zero previous norm gives a change of 0 when the norm is still zero
 * and +infinity otherwise.
 */
static void awp_layer_step(struct awp_layer_state *layer, double norm, double threshold,
                           int interval, int step_bits)
{
    double change;
    if (layer->previous_norm == 0.0)
        change = (norm == 0.0) ? 0.0 : (double)INFINITY;
    else
        change = (norm - layer->previous_norm) / layer->previous_norm;
    if (change < threshold)
        layer->counted += 1;
    if (layer->counted == interval) {
        layer->bits += step_bits;
        if (layer->bits > 32) layer->bits = 32;
        layer->counted = 0;
    }
}

/*
 * One batch of the AWP rule for all layers.  The first batch has no
 * predecessor and only records the norms.  The number of bytes sent for a
 * layer is its bit count rounded up to whole bytes (Section III-A: 14 bits ->
 * 2 bytes).  The arrays are the layers' states, kept by the caller.
 */
void oracle_awp_update(const double *l2_now, double *l2_prev, int32_t *counter,
                       int32_t *bits, uint8_t *bytes_out, int n_layers,
                       double T, int INTERVAL, int N, int is_first_batch)
{
    for (int layer = 0; layer < n_layers; ++layer) {
        struct awp_layer_state state = {l2_prev[layer], counter[layer], bits[layer]};
        if (!is_first_batch)
            awp_layer_step(&state, l2_now[layer], T, INTERVAL, N);
        state.previous_norm = l2_now[layer];
        l2_prev[layer] = state.previous_norm;
        counter[layer] = state.counted;
        bits[layer] = state.bits;
        bytes_out[layer] = (uint8_t)((state.bits + 7) / 8);
    }
}
