// Sanitizer driver for the host side of libadt (built by tests/test_sanitizers.py
// together with the library's sources, host code under -fsanitize=address,undefined).
// It only reaches code that runs before any GPU call: table validation, the byte
// count arithmetic, the scalar AWP rule, the group helpers, the tuning calls and
// the limits of the entry point that allocates nothing.  Buffers are heap blocks
// of exactly the size a call may touch.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "adt.h"
#include "adt_measure.h"

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            printf("check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main() {
    const std::vector<int64_t> sizes = {0, 1, 2, 3, 5, 15, 17, 4095, 0, 4097, 64, 0};
    const int L = (int)sizes.size();
    std::vector<int64_t> off(L + 1);
    std::vector<uint8_t> rb(L);
    int64_t n = 0, packed = 0;
    for (int l = 0; l < L; ++l) {
        off[l] = n;
        rb[l] = (uint8_t)(l % 2 ? 3 : 1);                         // 1,3,1,3,...
        n += sizes[l];
        packed += sizes[l] * rb[l];
    }
    off[L] = n;
    CHECK(adt_packed_size(off.data(), rb.data(), L) == packed);
    CHECK(adt_packed_size(off.data(), rb.data(), 0) == 0);
    float *fake = (float *)0x1000;                                 // never dereferenced
    uint8_t *fake8 = (uint8_t *)0x1000;
    {
        std::vector<uint8_t> bad(rb);
        bad[L - 1] = 5;
        CHECK(adt_packed_size(off.data(), bad.data(), L) == ADT_EINVAL);
        CHECK(adt_pack(fake, off.data(), bad.data(), L, fake8, nullptr) == ADT_EINVAL);
        CHECK(adt_unpack(fake8, off.data(), bad.data(), L, fake, nullptr) == ADT_EINVAL);
        CHECK(adt_pack_unpack(fake, off.data(), bad.data(), L, fake8, fake, nullptr) == ADT_EINVAL);
        CHECK(strlen(adt_last_error()) > 0);
        std::vector<int64_t> dec(off);
        dec[3] = dec[2] - 1;
        CHECK(adt_pack(fake, dec.data(), rb.data(), L, fake8, nullptr) == ADT_EINVAL);
        CHECK(awp_layer_stats(fake, dec.data(), L, (double *)fake, nullptr) == ADT_EINVAL);
        CHECK(adt_pack((const float *)0x1002, off.data(), rb.data(), L, fake8, nullptr) == ADT_EALIGN);
        CHECK(adt_unpack16(fake8, off.data(), rb.data(), L, (uint16_t *)fake, 7, nullptr) == ADT_EINVAL);
    }
    {   // only empty layers: success without a launch
        std::vector<int64_t> zero(4, 0);
        std::vector<uint8_t> r3 = {1, 3, 1};
        CHECK(adt_pack(nullptr, zero.data(), r3.data(), 3, nullptr, nullptr) == ADT_OK);
        CHECK(adt_unpack(nullptr, zero.data(), r3.data(), 3, nullptr, nullptr) == ADT_OK);
    }
    {   // the entry point that allocates nothing: limits are checked before the GPU is touched
        std::vector<int64_t> big = {0, (int64_t)8192 * AWP_NOALLOC_MAX_TILES + 1};
        CHECK(awp_layer_stats_noalloc(fake, big.data(), 1, (double *)fake, nullptr) == ADT_ERANGE);
        std::vector<int64_t> many(131);
        for (int i = 0; i < 131; ++i) many[i] = i;
        CHECK(awp_layer_stats_noalloc(fake, many.data(), 130, (double *)fake, nullptr) == ADT_ERANGE);
        CHECK(awp_layer_stats_noalloc(nullptr, many.data(), 0, nullptr, nullptr) == ADT_OK);
    }
    {   // the scalar rule against its definition (Algorithm 1), 60 batches
        const int G = 4;
        std::vector<double> now(G), prev(G, 0.0);
        std::vector<int32_t> counter(G, 0), bits = {8, 14, 31, 16};
        std::vector<uint8_t> bytes(G);
        std::vector<int32_t> e_counter(G, 0), e_bits(bits);
        std::vector<double> e_prev(G, 0.0);
        for (int b = 0; b < 60; ++b) {
            for (int g = 0; g < G; ++g) now[g] = g == 2 ? 0.0 : (b % 3 == g % 3 ? 2.0 : 1.0) * (g + 1);
            CHECK(awp_update(now.data(), prev.data(), counter.data(), bits.data(), bytes.data(), G,
                             -0.25, 3, 5, b == 0) == ADT_OK);
            for (int g = 0; g < G; ++g) {
                if (b > 0) {
                    const double d = e_prev[g] == 0.0 ? (now[g] == 0.0 ? 0.0 : INFINITY)
                                                      : (now[g] - e_prev[g]) / e_prev[g];
                    if (d < -0.25) ++e_counter[g];
                    if (e_counter[g] == 3) {
                        e_bits[g] = e_bits[g] + 5 > 32 ? 32 : e_bits[g] + 5;
                        e_counter[g] = 0;
                    }
                }
                e_prev[g] = now[g];
                CHECK(bits[g] == e_bits[g] && counter[g] == e_counter[g] && prev[g] == e_prev[g]);
                CHECK(bytes[g] == (bits[g] + 7) / 8);
            }
        }
        CHECK(awp_update(nullptr, prev.data(), counter.data(), bits.data(), bytes.data(), G, 0, 1, 8, 0) ==
              ADT_EINVAL);
        CHECK(awp_update(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, 1, 8, 0) == ADT_OK);
    }
    {   // group helpers
        std::vector<double> stats(3 * L);
        for (int l = 0; l < L; ++l) { stats[3 * l] = l * l; stats[3 * l + 1] = l; stats[3 * l + 2] = 1; }
        std::vector<int32_t> groups = {0, 3, 3, 9, L};
        std::vector<double> norms(4);
        CHECK(awp_group_norms(stats.data(), groups.data(), 4, norms.data()) == ADT_OK);
        CHECK(norms[0] == sqrt(0.0 + 1.0 + 4.0) && norms[1] == 0.0);
        std::vector<uint8_t> gb = {1, 2, 3, 4}, lb(L);
        CHECK(awp_expand_group_bytes(gb.data(), groups.data(), 4, lb.data()) == ADT_OK);
        CHECK(lb[0] == 1 && lb[2] == 1 && lb[3] == 3 && lb[8] == 3 && lb[9] == 4 && lb[L - 1] == 4);
        std::vector<int32_t> badg = {0, 5, 4, L};
        CHECK(awp_group_norms(stats.data(), badg.data(), 3, norms.data()) == ADT_EINVAL);
    }
    {   // plans are validated before anything is allocated
        awp_plan *plan = nullptr;
        std::vector<int64_t> dec = {0, 9, 8};
        CHECK(awp_plan_create(dec.data(), 2, nullptr, 0.0, 10, 8, &plan) == ADT_EINVAL && !plan);
        CHECK(awp_plan_create(off.data(), L, nullptr, 0.0, 0, 8, &plan) == ADT_EINVAL && !plan);
        std::vector<int32_t> groups = {0, 3};
        CHECK(awp_plan_create_grouped(off.data(), L, groups.data(), 1, nullptr, 0.0, 1, 8, &plan) ==
              ADT_EINVAL);
        CHECK(awp_adt_step(nullptr, fake, fake8, 0, fake, nullptr) == ADT_EINVAL);
        CHECK(awp_plan_destroy(nullptr) == ADT_OK);
    }
    {   // tuning calls
        int pack = -1, unpack = -1, stats_final = -1;
        for (int k = 0; k < ADT_NKERNELS; ++k) {
            if (!strcmp(adt_kernel_name(k), "pack_kernel")) pack = k;
            if (!strcmp(adt_kernel_name(k), "unpack_kernel")) unpack = k;
            if (!strcmp(adt_kernel_name(k), "stats_final_kernel")) stats_final = k;
        }
        CHECK(pack >= 0 && unpack >= 0 && stats_final >= 0 && adt_kernel_name(ADT_NKERNELS)[0] == 0);
        CHECK(adt_launch_shape(pack, 1, 4096) == ADT_OK && adt_launch_shape(pack, 0, 0) == ADT_OK);
        CHECK(adt_launch_shape(pack, 2, 0) == ADT_EINVAL && adt_launch_shape(unpack, 4, 0) == ADT_EINVAL);
        CHECK(adt_launch_shape(stats_final, 4, 0) == ADT_EINVAL && adt_launch_shape(pack, 1, 1 << 20) == ADT_EINVAL);
        const int64_t old = adt_stream_cache_limit(pack, -1);
        CHECK(old > 0 && adt_stream_cache_limit(pack, 123) == old && adt_stream_cache_limit(pack, old) == 123);
        CHECK(adt_stream_cache_limit(unpack, 0) == ADT_EINVAL);
        CHECK(adt_timing_enable(0, 0) == ADT_OK);
        CHECK(!strcmp(adt_strerror(ADT_ERANGE), "size out of range") && adt_source_digest() != nullptr);
    }
    printf("host sanitizer driver ok\n");
    return 0;
}
