// Optional in-kernel phase timestamps (development aid).  Compiled out unless the library is
// built with -DLSHBEAM_TRACE; then thread 0 of workgroup 0 of each kernel stores the 100 MHz
// wall clock at marked points into a device array that lsh_trace_read() copies out.
#pragma once
#include <hip/hip_runtime.h>

#ifdef LSHBEAM_TRACE
namespace lshbeam {
constexpr int kTraceKernels = 4, kTraceSlots = 16;
__device__ unsigned long long g_trace[kTraceKernels][kTraceSlots];
}
#define LSH_TRACE(kernel, slot)                                                   \
    do {                                                                          \
        if (blockIdx.x == 0 && threadIdx.x == 0)                                  \
            lshbeam::g_trace[kernel][slot] = wall_clock64();                      \
    } while (0)
#else
#define LSH_TRACE(kernel, slot) do { } while (0)
#endif
