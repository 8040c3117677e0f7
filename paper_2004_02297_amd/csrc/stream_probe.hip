// Streaming-rate probe for MI355X (gfx950): what does the chip sustain for the
// traffic mixes of the ADT / AWP kernels, independent of those kernels?
//
// Bare kernels over 138,344,128 FP32 words (the VGG-16-shaped weight count):
// pure read, pure write, copy, two reads per write (pack-like) and one read per
// two writes (unpack-like), each with ordinary and with nontemporal accesses,
// and each with the number of blocks a compute unit may hold lowered through
// unused dynamic LDS.  Prints one line per case: microseconds per launch
// (30 back-to-back launches between two HIP events), GB/s and the fraction of
// the 8 TB/s HBM peak.  The library's cache hints and occupancy caps were chosen
// from these numbers.
//
// Build: hipcc --offload-arch=gfx950 -O3 -o stream_probe stream_probe.hip
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4 *p) {
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void st(u32x4 *p, u32x4 v) {
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Every block of 256 threads moves 1024 vectors of 16 bytes on its widest side.
template <bool NT>
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ in,
                                                   uint32_t *__restrict__ sink) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = ld<NT>(in + base + j * 256);
    uint32_t a = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) a ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    if (a == 0x12345678u) sink[blockIdx.x] = a;     // keeps the loads alive
}

template <bool NT>
__global__ __launch_bounds__(256) void write_kernel(u32x4 *__restrict__ out) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    const u32x4 v = {1u, 2u, 3u, (uint32_t)base};
#pragma unroll
    for (int j = 0; j < 4; ++j) st<NT>(out + base + j * 256, v);
}

template <bool NTL, bool NTS>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ in,
                                                   u32x4 *__restrict__ out) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = ld<NTL>(in + base + j * 256);
#pragma unroll
    for (int j = 0; j < 4; ++j) st<NTS>(out + base + j * 256, v[j]);
}

template <bool NTL, bool NTS>
__global__ __launch_bounds__(256) void two_reads_one_write(const u32x4 *__restrict__ in,
                                                           u32x4 *__restrict__ out) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = ld<NTL>(in + base + j * 256);
    st<NTS>(out + (size_t)blockIdx.x * 512 + threadIdx.x, v[0] ^ v[1]);
    st<NTS>(out + (size_t)blockIdx.x * 512 + 256 + threadIdx.x, v[2] ^ v[3]);
}

template <bool NTL, bool NTS>
__global__ __launch_bounds__(256) void one_read_two_writes(const u32x4 *__restrict__ in,
                                                           u32x4 *__restrict__ out) {
    const size_t base = (size_t)blockIdx.x * 512 + threadIdx.x;
    const u32x4 a = ld<NTL>(in + base), b = ld<NTL>(in + base + 256);
    const size_t o = (size_t)blockIdx.x * 1024 + threadIdx.x;
    st<NTS>(out + o, a);
    st<NTS>(out + o + 256, b);
    st<NTS>(out + o + 512, a ^ b);
    st<NTS>(out + o + 768, a + b);
}

static const int kIters = 30;

template <typename Launch>
static int run(const char *name, double bytes, unsigned lds_kb, Launch launch) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i) launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, 0));
    for (int i = 0; i < kIters; ++i) launch();
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipGetLastError());
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    ms /= kIters;
    printf("%-34s blocks/CU<=%-2u %8.1f us %7.0f GB/s  %.3f of 8 TB/s\n", name,
           lds_kb ? 160u / lds_kb : 8u, ms * 1e3, bytes / ms / 1e6, bytes / ms / 1e6 / 8000.0);
    fflush(stdout);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

template <typename K>
static int allow_big_lds(K kernel) {
    CHECK(hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024));
    return 0;
}

int main() {
    const size_t N = 138344128;          // FP32 words
    const size_t n4 = N / 4;             // 16-byte vectors
    const unsigned grid = (unsigned)(n4 / 1024);
    u32x4 *in = nullptr, *out = nullptr;
    uint32_t *sink = nullptr;
    CHECK(hipMalloc(&in, N * 4));
    CHECK(hipMalloc(&out, N * 4));
    CHECK(hipMalloc(&sink, (size_t)grid * 4));
    CHECK(hipMemset(in, 1, N * 4));
    CHECK(hipMemset(out, 0, N * 4));
    const double B = 4.0 * (double)grid * 1024 * 4;   // bytes of one full pass over the words

    if (allow_big_lds(read_kernel<true>) || allow_big_lds(read_kernel<false>) ||
        allow_big_lds(write_kernel<true>) || allow_big_lds(write_kernel<false>) ||
        allow_big_lds(copy_kernel<true, true>) || allow_big_lds(copy_kernel<false, false>) ||
        allow_big_lds(two_reads_one_write<true, true>) ||
        allow_big_lds(two_reads_one_write<true, false>) ||
        allow_big_lds(two_reads_one_write<false, false>) ||
        allow_big_lds(one_read_two_writes<true, true>) ||
        allow_big_lds(one_read_two_writes<false, false>))
        return 1;

    // dynamic LDS per block in KB: 0 -> 8 blocks (32 waves) per CU, 32 -> 5, 40 -> 4, 53 -> 3, 80 -> 2
    const unsigned caps[] = {0, 32, 40, 53, 80};
    for (unsigned kb : caps) {
        const unsigned lds = kb * 1024;
        int rc = 0;
        rc |= run("read, ordinary loads", B, kb, [&] { read_kernel<false><<<grid, 256, lds>>>(in, sink); });
        rc |= run("read, nontemporal loads", B, kb, [&] { read_kernel<true><<<grid, 256, lds>>>(in, sink); });
        rc |= run("write, ordinary stores", B, kb, [&] { write_kernel<false><<<grid, 256, lds>>>(out); });
        rc |= run("write, nontemporal stores", B, kb, [&] { write_kernel<true><<<grid, 256, lds>>>(out); });
        rc |= run("copy, ordinary", 2 * B, kb, [&] { copy_kernel<false, false><<<grid, 256, lds>>>(in, out); });
        rc |= run("copy, nontemporal", 2 * B, kb, [&] { copy_kernel<true, true><<<grid, 256, lds>>>(in, out); });
        rc |= run("2 reads : 1 write, ordinary", 1.5 * B, kb,
                  [&] { two_reads_one_write<false, false><<<grid, 256, lds>>>(in, out); });
        rc |= run("2 reads : 1 write, nt loads only", 1.5 * B, kb,
                  [&] { two_reads_one_write<true, false><<<grid, 256, lds>>>(in, out); });
        rc |= run("2 reads : 1 write, nontemporal", 1.5 * B, kb,
                  [&] { two_reads_one_write<true, true><<<grid, 256, lds>>>(in, out); });
        rc |= run("1 read : 2 writes, ordinary", 1.5 * B, kb,
                  [&] { one_read_two_writes<false, false><<<grid, 256, lds>>>(in, out); });
        rc |= run("1 read : 2 writes, nontemporal", 1.5 * B, kb,
                  [&] { one_read_two_writes<true, true><<<grid, 256, lds>>>(in, out); });
        if (rc) return 1;
    }
    int rc = run("hipMemcpyAsync device to device", 2 * B, 0, [&] {
        (void)hipMemcpyAsync(out, in, (size_t)grid * 1024 * 16, hipMemcpyDeviceToDevice, 0);
    });
    (void)hipFree(in);
    (void)hipFree(out);
    (void)hipFree(sink);
    return rc;
}
