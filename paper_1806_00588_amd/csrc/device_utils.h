// Wave64 / workgroup helpers shared by the lshbeam kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lshbeam {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        uint32_t n = __shfl_up(v, off, kWave);
        if (lane_id() >= off) v += n;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Order-preserving map fp32 -> uint32 (larger float <=> larger integer; -0 is folded into +0 by
// the caller adding 0.0f first).
__device__ __forceinline__ uint32_t f32_sortable(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float sortable_f32(uint32_t s) {
    uint32_t u = (s & 0x80000000u) ? (s & 0x7FFFFFFFu) : ~s;
    return __uint_as_float(u);
}

// Element loads: fp32 as is, bf16 bit patterns widened exactly (the stored 16 bits are the top
// half of the fp32 pattern).
__device__ __forceinline__ float elem_f32(const float* p) { return *p; }
__device__ __forceinline__ float elem_f32(const uint16_t* p) {
    return __uint_as_float((uint32_t)(*p) << 16);
}

// Workgroup inclusive scan; `wsum` is LDS with at least blockDim.x/64 + 1 words.  Returns the
// inclusive prefix of v for this thread and the workgroup total in *total.  Ends with a barrier,
// so wsum may be reused right after.
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wsum, uint32_t* total) {
    const int nw = blockDim.x >> 6;
    uint32_t incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) wsum[wave_id()] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (int w = 0; w < nw; ++w) {
        uint32_t x = wsum[w];
        if (w < wave_id()) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return incl + base;
}

}  // namespace lshbeam
