// Kernel launch helper shared by the launchers: an ordinary launch, or, while
// launch timing is switched on (adt_timing_enable), a launch bracketed by the
// dispatch's own begin / end timestamps (hipExtLaunchKernel events), so that a
// benchmark reads exact kernel durations without a profiler attached.
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adt_tables.h"

namespace adt {

enum KernelId {
    kKernelPack = 0,
    kKernelUnpack = 1,
    kKernelStatsPartial = 2,
    kKernelStatsFinal = 3,
    kKernelFused = 4,
    kKernelFinalRule = 5,
    kKernelRedo = 6,
    kKernelPackUnpack = 7,
    kKernelUnpack16 = 8,
    kKernelPrefix = 9,
    kNumKernels = 10
};

// Defined in adt_api.hip.  True (and a fresh event pair, owned by the timing
// registry) when launch timing is on and `stream` is not being captured into a
// graph (a captured launch is an ordinary launch: timing events would never
// complete).
bool timing_events(int kernel_id, hipStream_t stream, hipEvent_t *start, hipEvent_t *stop);

// extra_lds: bytes of dynamic LDS the kernel does not use; they only lower
// the number of blocks a compute unit holds at once.
template <typename Args>
hipError_t launch(void (*kernel)(Args), int kernel_id, uint32_t grid, int block,
                  hipStream_t stream, const Args &args, uint32_t extra_lds = 0) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (timing_events(kernel_id, stream, &e0, &e1))
        hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(block), extra_lds, stream, e0, e1, 0, args);
    else
        kernel<<<dim3(grid), dim3(block), extra_lds, stream>>>(args);
    return hipGetLastError();
}

}  // namespace adt
