/*
 * A plain C program that drives libadt on the GPU with no Python in between:
 * reads the Tiny case and the CPU oracle's results from tests/golden/tiny_case.bin
 * (written by tests/golden/make_tiny_case.py), allocates device memory with the
 * HIP C API, calls adt_pack, adt_unpack, adt_pack_unpack, awp_layer_stats and
 * awp_layer_stats_noalloc, and compares: stream and unpacked words bit for bit,
 * statistics to 1e-10 relative (largest magnitude exactly).
 * usage: gpu_client path/to/tiny_case.bin
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adt.h"

#define HIP(x)                                                                      \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 2;                                                               \
        }                                                                           \
    } while (0)
#define ADT(x)                                                                      \
    do {                                                                            \
        int s_ = (x);                                                               \
        if (s_ != ADT_OK) {                                                         \
            printf("libadt %s (%s) at line %d\n", adt_strerror(s_), adt_last_error(), __LINE__); \
            return 3;                                                               \
        }                                                                           \
    } while (0)
#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            printf("check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                 \
        }                                                             \
    } while (0)

static size_t pad8(size_t n) { return (n + 7) & ~(size_t)7; }

static int stats_match(const double *got, const double *exp, int n_layers) {
    for (int l = 0; l < n_layers; ++l) {
        for (int k = 0; k < 2; ++k) {
            const double g = got[3 * l + k], e = exp[3 * l + k];
            if (fabs(g - e) > 1e-10 * fabs(e)) return 0;
        }
        if (got[3 * l + 2] != exp[3 * l + 2]) return 0;
    }
    return 1;
}

int main(int argc, char **argv) {
    if (argc < 2) return 64;
    FILE *f = fopen(argv[1], "rb");
    if (!f) { printf("cannot open %s\n", argv[1]); return 65; }
    fseek(f, 0, SEEK_END);
    const long size = ftell(f);
    fseek(f, 0, SEEK_SET);
    unsigned char *blob = (unsigned char *)malloc((size_t)size);
    if (fread(blob, 1, (size_t)size, f) != (size_t)size) return 66;
    fclose(f);
    CHECK(memcmp(blob, "ADTT", 4) == 0);
    int32_t L;
    memcpy(&L, blob + 4, 4);
    const int64_t *off = (const int64_t *)(blob + 8);
    const uint8_t *rb = blob + 8 + 8 * (size_t)(L + 1);
    size_t at = 8 + 8 * (size_t)(L + 1) + pad8((size_t)L);
    int64_t packed;
    memcpy(&packed, blob + at, 8);
    at += 8;
    const int64_t n = off[L];
    const float *weights = (const float *)(blob + at);
    at += 4 * (size_t)n;
    const uint8_t *exp_stream = blob + at;
    at += pad8((size_t)packed);
    const float *exp_unpacked = (const float *)(blob + at);
    at += 4 * (size_t)n;
    const double *exp_stats = (const double *)(blob + at);
    CHECK(at + 24 * (size_t)L == (size_t)size);
    CHECK(adt_packed_size(off, rb, L) == packed);

    float *d_w, *d_back, *d_back2;
    uint8_t *d_p, *d_p2;
    double *d_stats, *d_stats2;
    HIP(hipMalloc((void **)&d_w, 4 * (size_t)n));
    HIP(hipMalloc((void **)&d_back, 4 * (size_t)n));
    HIP(hipMalloc((void **)&d_back2, 4 * (size_t)n));
    HIP(hipMalloc((void **)&d_p, (size_t)packed));
    HIP(hipMalloc((void **)&d_p2, (size_t)packed));
    HIP(hipMalloc((void **)&d_stats, 24 * (size_t)L));
    HIP(hipMalloc((void **)&d_stats2, 24 * (size_t)L));
    HIP(hipMemcpy(d_w, weights, 4 * (size_t)n, hipMemcpyHostToDevice));
    HIP(hipMemset(d_p, 0xA5, (size_t)packed));
    HIP(hipMemset(d_back, 0x5A, 4 * (size_t)n));
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));

    ADT(awp_layer_stats(d_w, off, L, d_stats, stream));
    ADT(awp_layer_stats_noalloc(d_w, off, L, d_stats2, stream));
    ADT(adt_pack(d_w, off, rb, L, d_p, stream));
    ADT(adt_unpack(d_p, off, rb, L, d_back, stream));
    ADT(adt_pack_unpack(d_w, off, rb, L, d_p2, d_back2, stream));
    HIP(hipStreamSynchronize(stream));

    uint8_t *h_p = (uint8_t *)malloc((size_t)packed);
    float *h_back = (float *)malloc(4 * (size_t)n);
    double *h_stats = (double *)malloc(24 * (size_t)L);
    HIP(hipMemcpy(h_p, d_p, (size_t)packed, hipMemcpyDeviceToHost));
    CHECK(memcmp(h_p, exp_stream, (size_t)packed) == 0);
    HIP(hipMemcpy(h_p, d_p2, (size_t)packed, hipMemcpyDeviceToHost));
    CHECK(memcmp(h_p, exp_stream, (size_t)packed) == 0);
    HIP(hipMemcpy(h_back, d_back, 4 * (size_t)n, hipMemcpyDeviceToHost));
    CHECK(memcmp(h_back, exp_unpacked, 4 * (size_t)n) == 0);
    HIP(hipMemcpy(h_back, d_back2, 4 * (size_t)n, hipMemcpyDeviceToHost));
    CHECK(memcmp(h_back, exp_unpacked, 4 * (size_t)n) == 0);
    HIP(hipMemcpy(h_stats, d_stats, 24 * (size_t)L, hipMemcpyDeviceToHost));
    CHECK(stats_match(h_stats, exp_stats, L));
    HIP(hipMemcpy(h_stats, d_stats2, 24 * (size_t)L, hipMemcpyDeviceToHost));
    CHECK(stats_match(h_stats, exp_stats, L));

    ADT(adt_shutdown());
    HIP(hipStreamDestroy(stream));
    HIP(hipFree(d_w)); HIP(hipFree(d_back)); HIP(hipFree(d_back2)); HIP(hipFree(d_p));
    HIP(hipFree(d_p2)); HIP(hipFree(d_stats)); HIP(hipFree(d_stats2));
    printf("c client ok: %d layers, %lld weights, %lld stream bytes\n", (int)L, (long long)n,
           (long long)packed);
    return 0;
}
