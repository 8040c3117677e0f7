/*
 * Sanitizer driver for the CPU oracle (built with -fsanitize=address,undefined
 * by tests/test_sanitizers.py).  Every buffer is a heap block of exactly the
 * size the call may touch, so that an access one byte outside is reported.
 * Edge tables: empty layers, byte counts 1,3,1,3,..., ragged sizes.
 * Exit status 0 = all checks passed and the sanitizers stayed silent.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_pack(const float *W, const int64_t *layer_offsets, const uint8_t *bytes_per_layer,
                    int n_layers, uint8_t *Pw);
int64_t oracle_unpack(const uint8_t *Pw, const int64_t *layer_offsets,
                      const uint8_t *bytes_per_layer, int n_layers, float *W);
void oracle_stats(const float *W, const int64_t *layer_offsets, int n_layers, double *stats);
void oracle_group_norms(const float *W, const int64_t *layer_offsets, const int32_t *group_offsets,
                        int n_groups, double *l2_group);
void oracle_awp_update(const double *l2_now, double *l2_prev, int32_t *counter, int32_t *bits,
                       uint8_t *bytes_out, int n_layers, double T, int INTERVAL, int N,
                       int is_first_batch);

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            printf("check failed at line %d: %s\n", __LINE__, #cond);      \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static uint32_t next_word(uint32_t *s) {           /* any bit pattern, NaN and Inf included */
    *s = *s * 1664525u + 1013904223u;
    return *s ^ (*s >> 13);
}

int main(void) {
    const int64_t sizes[] = {0, 1, 2, 3, 5, 15, 17, 4095, 0, 4097, 64, 0};
    const int L = (int)(sizeof(sizes) / sizeof(sizes[0]));
    int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
    uint8_t *rb = (uint8_t *)malloc((size_t)L);
    int64_t n = 0, packed = 0;
    for (int l = 0; l < L; ++l) {
        off[l] = n;
        rb[l] = (uint8_t)(l % 4 == 3 ? 4 : (l % 2 ? 3 : 1));      /* 1,3,1,4,1,3,1,4,... */
        if (l == 6) rb[l] = 2;
        n += sizes[l];
        packed += sizes[l] * rb[l];
    }
    off[L] = n;

    uint32_t *words = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    uint32_t seed = 12345u;
    for (int64_t i = 0; i < n; ++i) words[i] = next_word(&seed);
    uint8_t *stream = (uint8_t *)malloc((size_t)packed);
    uint32_t *back = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    CHECK(oracle_pack((const float *)words, off, rb, L, stream) == packed);
    CHECK(oracle_unpack(stream, off, rb, L, (float *)back) == packed);
    for (int l = 0; l < L; ++l) {
        const uint32_t mask = rb[l] == 4 ? 0xFFFFFFFFu : 0xFFFFFFFFu << (8 * (4 - rb[l]));
        for (int64_t i = off[l]; i < off[l + 1]; ++i) CHECK(back[i] == (words[i] & mask));
    }
    /* invalid tables are refused without touching the buffers */
    uint8_t bad[2] = {2, 5};
    int64_t two[3] = {0, 1, 2};
    CHECK(oracle_pack((const float *)words, two, bad, 2, stream) == -1);
    CHECK(oracle_unpack(stream, two, bad, 2, (float *)back) == -1);
    /* no layers at all, null data pointers */
    int64_t none[1] = {0};
    CHECK(oracle_pack(NULL, none, NULL, 0, NULL) == 0);

    /* statistics on finite values (ragged + empty layers) */
    float *w = (float *)malloc(sizeof(float) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) w[i] = (float)((int)(next_word(&seed) % 2001) - 1000) * 1e-3f;
    double *stats = (double *)malloc(sizeof(double) * 3 * (size_t)L);
    oracle_stats(w, off, L, stats);
    for (int l = 0; l < L; ++l) {
        double s = 0.0, m = 0.0;
        for (int64_t i = off[l]; i < off[l + 1]; ++i) {
            s += (double)w[i] * (double)w[i];
            if (fabs((double)w[i]) > m) m = fabs((double)w[i]);
        }
        CHECK(stats[3 * l] == s && stats[3 * l + 1] == sqrt(s) && stats[3 * l + 2] == m);
    }
    int32_t groups[5] = {0, 3, 3, 9, L};
    double norms[4];
    oracle_group_norms(w, off, groups, 4, norms);
    CHECK(norms[1] == 0.0);
    {
        double s = 0.0;
        for (int l = 3; l < 9; ++l) s += stats[3 * l];
        CHECK(fabs(norms[2] - sqrt(s)) <= 1e-12 * norms[2]);
    }

    /* AWP rule: 40 batches, upgrades every 2 counted batches, cap at 32 bits */
    double now[3], prev[3] = {0, 0, 0};
    int32_t counter[3] = {0, 0, 0}, bits[3] = {8, 14, 31};
    uint8_t bytes[3];
    for (int b = 0; b < 40; ++b) {
        for (int l = 0; l < 3; ++l) now[l] = l == 2 ? 0.0 : 10.0 / (1.0 + b);   /* shrinking, and a zero norm */
        oracle_awp_update(now, prev, counter, bits, bytes, 3, 0.0, 2, 8, b == 0);
        for (int l = 0; l < 3; ++l) CHECK(bytes[l] == (bits[l] + 7) / 8 && bits[l] <= 32);
    }
    CHECK(bits[0] == 32 && bits[1] == 32 && bits[2] == 31 && counter[2] == 0);

    free(off); free(rb); free(words); free(stream); free(back); free(w); free(stats);
    printf("oracle sanitizer driver ok: %lld weights, %lld packed bytes\n", (long long)n, (long long)packed);
    return 0;
}
