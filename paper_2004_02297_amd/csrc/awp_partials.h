// Fixed-order reduction of per-tile statistics partials to per-layer statistics
// (Section II of arXiv 2004.02297: the l2-norm of all weights of a layer), shared
// by the final kernel of awp_layer_stats and by the plan's final reduction + rule.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_tables.h"

namespace adt {

constexpr int kFinalBlock = 1024;
constexpr int kFinalWaves = kFinalBlock / kWave;

// Wave-wide reductions without LDS traffic: four data-parallel-primitive steps
// inside every row of 16 lanes (swap neighbours, swap pairs, mirror within 8,
// mirror within 16: after each step the lanes of a group all hold the group's
// value, because both partners compute the same commutative operation), then
// the four row values are read with v_readlane and combined as
// (r0 + r1) + (r2 + r3).  All 64 lanes must be active.  Every lane returns the
// same value, and the order of the additions is fixed.
constexpr int kDppSwap1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within 16

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint32_t lo = dpp_u32<CTRL>((uint32_t)__double2loint(v));
    const uint32_t hi = dpp_u32<CTRL>((uint32_t)__double2hiint(v));
    return __hiloint2double((int)hi, (int)lo);
}

__device__ __forceinline__ double lane_f64(double v, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_f64<kDppSwap1>(v);
    v += dpp_f64<kDppSwap2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppMirror>(v);
    return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
    v = umax(v, dpp_u32<kDppSwap1>(v));
    v = umax(v, dpp_u32<kDppSwap2>(v));
    v = umax(v, dpp_u32<kDppHalfMirror>(v));
    v = umax(v, dpp_u32<kDppMirror>(v));
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
    const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return umax(umax(r0, r1), umax(r2, r3));
}

// Magnitude bits: ordering them as unsigned integers orders finite values and
// infinity by magnitude and puts every NaN above infinity, so a NaN wins.
__device__ __forceinline__ void square_add(uint32_t bits, double &acc, uint32_t &mag) {
    const double w = (double)__uint_as_float(bits);
    acc = fma(w, w, acc);               // the square of a binary32 is exact in binary64
    const uint32_t m = bits & 0x7FFFFFFFu;
    mag = m > mag ? m : mag;
}

// One wavefront adds partials [begin, end) in an order fixed by the indices
// alone: lane t takes begin+t, begin+t+64, ... (eight loads in flight per
// round), then the lanes are combined by wave_sum / wave_max.  Every lane
// returns the result.  All 64 lanes must be active.  COHERENT: the partials were
// handed over by other blocks of the same launch through device-scope atomic
// exchanges and are read with device-scope atomic loads (no cache in between).
template <bool COHERENT = false>
__device__ __forceinline__ void wave_reduce_partials(const double *partial_sumsq,
                                                     const uint32_t *partial_absmax,
                                                     uint32_t begin, uint32_t end, int lane,
                                                     double &sumsq, uint32_t &magnitude) {
    constexpr int kInFlight = 8;
    double acc = 0.0;
    uint32_t mag = 0u;
    for (uint32_t base = begin; base < end; base += kInFlight * kWave) {   // wave uniform
        double v[kInFlight];
        uint32_t m[kInFlight];
#pragma unroll
        for (int j = 0; j < kInFlight; ++j) {
            const uint32_t k = base + (uint32_t)(j * kWave + lane);
            const bool ok = k < end;
            if (COHERENT) {
                v[j] = 0.0;
                m[j] = 0u;
                if (ok) {
                    v[j] = __longlong_as_double((long long)__hip_atomic_load(
                        (const unsigned long long *)(partial_sumsq + k), __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT));
                    m[j] = __hip_atomic_load(partial_absmax + k, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
                }
            } else {
                v[j] = ok ? partial_sumsq[k] : 0.0;
                m[j] = ok ? partial_absmax[k] : 0u;
            }
        }
#pragma unroll
        for (int j = 0; j < kInFlight; ++j) {
            acc += v[j];
            mag = m[j] > mag ? m[j] : mag;
        }
    }
    sumsq = wave_sum(acc);
    magnitude = wave_max(mag);
}

// One block of kFinalBlock threads adds partials [begin, end) in an order fixed
// by the indices alone: thread t takes begin+t, begin+t+1024, ... (sixteen loads
// in flight per round), a wave combines its lanes with xor-shuffles, thread 0
// adds the 16 wave sums in index order.  The result is valid in thread 0 only.
// Ends with a block barrier, so it may be called again right away.
__device__ __forceinline__ void reduce_partials(const double *__restrict__ partial_sumsq,
                                                const uint32_t *__restrict__ partial_absmax,
                                                uint32_t begin, uint32_t end, double &sumsq,
                                                uint32_t &magnitude) {
    __shared__ double wsum[kFinalWaves];
    __shared__ uint32_t wmag[kFinalWaves];
    constexpr int kInFlight = 16;
    double acc = 0.0;
    uint32_t mag = 0u;
    for (uint32_t i = begin + threadIdx.x; i < end; i += kInFlight * kFinalBlock) {
        double v[kInFlight];
        uint32_t m[kInFlight];
#pragma unroll
        for (int j = 0; j < kInFlight; ++j) {
            const uint32_t k = i + j * kFinalBlock;
            const bool ok = k < end;
            v[j] = ok ? partial_sumsq[k] : 0.0;
            m[j] = ok ? partial_absmax[k] : 0u;
        }
#pragma unroll
        for (int j = 0; j < kInFlight; ++j) {
            acc += v[j];
            mag = m[j] > mag ? m[j] : mag;
        }
    }
    acc = wave_sum(acc);
    mag = wave_max(mag);
    if ((threadIdx.x & 63) == 0) {
        wsum[threadIdx.x >> 6] = acc;
        wmag[threadIdx.x >> 6] = mag;
    }
    __syncthreads();
    double tot = 0.0;
    uint32_t tm = 0u;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < kFinalWaves; ++i) {
            tot += wsum[i];
            tm = wmag[i] > tm ? wmag[i] : tm;
        }
    }
    __syncthreads();
    sumsq = tot;
    magnitude = tm;
}

}  // namespace adt
