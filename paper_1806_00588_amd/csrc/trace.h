// Optional in-kernel phase timestamps (development aid).  Compiled out unless the library is
// built with -DLSHBEAM_TRACE; then thread 0 of workgroup 0 of each kernel stores the 100 MHz
// wall clock at marked points into a device array that lsh_trace_read() copies out
// (LSH_TRACE_LATEST: the latest time over all workgroups of the launch).
#pragma once
#include <hip/hip_runtime.h>

#ifdef LSHBEAM_TRACE
namespace lshbeam {
constexpr int kTraceKernels = 4, kTraceSlots = 16;
__device__ unsigned long long g_trace[kTraceKernels][kTraceSlots];
constexpr int kTraceWgs = 512, kTraceWgSlots = 8;
__device__ unsigned long long g_trace_wg[kTraceWgs][kTraceWgSlots];  // per workgroup (one kernel)
}
#define LSH_TRACE(kernel, slot)                                                   \
    do {                                                                          \
        if (blockIdx.x == 0 && threadIdx.x == 0)                                  \
            lshbeam::g_trace[kernel][slot] = wall_clock64();                      \
    } while (0)
// thread 0 of whichever workgroup passes (for code only one workgroup of a launch runs)
#define LSH_TRACE_ANY(kernel, slot)                                               \
    do {                                                                          \
        if (threadIdx.x == 0) lshbeam::g_trace[kernel][slot] = wall_clock64();    \
    } while (0)
// the latest time any workgroup of the launch passes the point
#define LSH_TRACE_LATEST(kernel, slot)                                            \
    do {                                                                          \
        if (threadIdx.x == 0) atomicMax(&lshbeam::g_trace[kernel][slot], wall_clock64()); \
    } while (0)
// thread 0 of every workgroup (of the one kernel that uses this macro)
#define LSH_TRACE_WG(slot)                                                        \
    do {                                                                          \
        if (threadIdx.x == 0 && blockIdx.x < lshbeam::kTraceWgs)                  \
            lshbeam::g_trace_wg[blockIdx.x][slot] = wall_clock64();               \
    } while (0)
// Development builds only: copy the phase timestamps (100 MHz ticks) to the host.
extern "C" __attribute__((used)) int lsh_trace_read(unsigned long long* out_host) {
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    return hipMemcpyFromSymbol(out_host, HIP_SYMBOL(lshbeam::g_trace),
                               sizeof(unsigned long long) * lshbeam::kTraceKernels * lshbeam::kTraceSlots) != hipSuccess;
}
extern "C" __attribute__((used)) int lsh_trace_read_wg(unsigned long long* out_host) {
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    return hipMemcpyFromSymbol(out_host, HIP_SYMBOL(lshbeam::g_trace_wg),
                               sizeof(unsigned long long) * lshbeam::kTraceWgs * lshbeam::kTraceWgSlots) != hipSuccess;
}
#else
#define LSH_TRACE_WG(slot) do { } while (0)
#define LSH_TRACE_ANY(kernel, slot) do { } while (0)
#define LSH_TRACE(kernel, slot) do { } while (0)
#define LSH_TRACE_LATEST(kernel, slot) do { } while (0)
#endif
