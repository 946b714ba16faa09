// Wave64 / workgroup helpers shared by the lshbeam kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "trace.h"

namespace lshbeam {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// DPP lane permutations (no LDS round trip, unlike ds_bpermute-based shuffles).
//   0x110 + n : row_shr:n   -- shift right by n lanes inside each row of 16 lanes
//   0x142     : row_bcast:15 -- lane 15 of each row to every lane of the next row
//   0x143     : row_bcast:31 -- lane 31 to every lane of rows 2 and 3
// Lanes that receive nothing (shifted in from outside the row, or rows disabled by row_mask)
// read `old` = 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}

// Inclusive prefix sum over the 64 lanes of a wave: Hillis-Steele inside each row of 16 lanes,
// then the row totals are carried across rows with the two broadcast steps.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    v += dpp_or_zero<0x111, 0xf>(v);
    v += dpp_or_zero<0x112, 0xf>(v);
    v += dpp_or_zero<0x114, 0xf>(v);
    v += dpp_or_zero<0x118, 0xf>(v);
    v += dpp_or_zero<0x142, 0xa>(v);  // rows 1 and 3 add the total of rows 0 and 2
    v += dpp_or_zero<0x143, 0xc>(v);  // rows 2 and 3 add the total of lanes 0..31
    return v;
}

// OR of v over the 64 lanes (same data movement as the scan; valid in lane 63, returned uniform).
__device__ __forceinline__ uint32_t wave_or(uint32_t v);

// Value of lane `lane` (compile-time or wave-uniform) broadcast through a scalar register.
__device__ __forceinline__ uint32_t wave_read_lane(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// Position of this lane among the set lanes of a ballot mask.
__device__ __forceinline__ uint32_t lanes_below(uint64_t bal) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
    return wave_read_lane(wave_incl_scan(v), kWave - 1);
}

__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
    v |= dpp_or_zero<0x111, 0xf>(v);
    v |= dpp_or_zero<0x112, 0xf>(v);
    v |= dpp_or_zero<0x114, 0xf>(v);
    v |= dpp_or_zero<0x118, 0xf>(v);
    v |= dpp_or_zero<0x142, 0xa>(v);
    v |= dpp_or_zero<0x143, 0xc>(v);
    return wave_read_lane(v, kWave - 1);
}

// Wave-wide float reductions on the DPP network (same data movement as the scan: valid in lane
// 63, returned wave-uniform).  Lanes that receive nothing keep the identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32_or(float v, float identity) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v),
                                                      CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_max_f32(float v) {
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_f32_or<0x111, 0xf>(v, ninf));
    v = fmaxf(v, dpp_f32_or<0x112, 0xf>(v, ninf));
    v = fmaxf(v, dpp_f32_or<0x114, 0xf>(v, ninf));
    v = fmaxf(v, dpp_f32_or<0x118, 0xf>(v, ninf));
    v = fmaxf(v, dpp_f32_or<0x142, 0xa>(v, ninf));
    v = fmaxf(v, dpp_f32_or<0x143, 0xc>(v, ninf));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}
__device__ __forceinline__ float wave_sum_f32(float v) {
    v += dpp_f32_or<0x111, 0xf>(v, 0.f);
    v += dpp_f32_or<0x112, 0xf>(v, 0.f);
    v += dpp_f32_or<0x114, 0xf>(v, 0.f);
    v += dpp_f32_or<0x118, 0xf>(v, 0.f);
    v += dpp_f32_or<0x142, 0xa>(v, 0.f);
    v += dpp_f32_or<0x143, 0xc>(v, 0.f);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}

// All-reduce inside each group of 16 consecutive lanes (a DPP "row"): xor-1 and xor-2 inside
// quads, then the half-row and full-row mirrors.  Every lane of the group ends with the result.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));   // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f32<0x4E>(v));   // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f32<0x141>(v));  // row_half_mirror
    v = fmaxf(v, dpp_f32<0x140>(v));  // row_mirror
    return v;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f32<0xB1>(v);
    v += dpp_f32<0x4E>(v);
    v += dpp_f32<0x141>(v);
    v += dpp_f32<0x140>(v);
    return v;
}

__device__ __forceinline__ int row16_min_i32(int v) {
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true));
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

// Stores that other workgroups of the SAME kernel will read (the one-launch plan's last workgroup
// reads what the others computed): device-scope atomic stores, which go through to memory instead
// of staying dirty in the L2 of the writer's XCD -- the eight XCDs' L2s are not coherent with each
// other inside a kernel.  Publishing then needs no cache write-back: wait for the stores to
// complete (publish_wait), barrier, ticket.  `AGENT` = false gives plain stores (the data is only
// read by a later kernel).
template <bool AGENT, typename T>
__device__ __forceinline__ void store_shared_result(T* p, T v) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit values");
    if constexpr (AGENT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
// All of this wave's stores have completed (been acknowledged by the memory they went through to).
__device__ __forceinline__ void publish_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// x / y for 0 <= x < 1024 and 1 <= y <= 1024 (thread indices by runtime table shapes) with four
// vector instructions instead of the ~25 of an integer division: (x + 0.5) / y is at least
// 0.5 / 1024 away from every integer, the float product errs by far less.
__device__ __forceinline__ int small_div(int x, int y) {
    return (int)(((float)x + 0.5f) * __builtin_amdgcn_rcpf((float)y));   // (v_rcp_f32: 1 ulp, ample here)
}

// Position of the r-th set bit (r = 0 for the lowest) of a word that has more than r bits set: a
// five-step search over popcounts of the low halves.
__host__ __device__ __forceinline__ uint32_t nth_set_bit(uint32_t bits, uint32_t r) {
    uint32_t at = 0;
#pragma unroll
    for (int half = 16; half >= 1; half >>= 1) {
        const uint32_t low = bits & ((1u << half) - 1u);
        const uint32_t c = (uint32_t)__builtin_popcount(low);
        if (r >= c) { r -= c; bits >>= half; at += half; } else { bits = low; }
    }
    return at;
}

// Workgroup barrier for data that is exchanged through LDS only: waits for this wave's LDS
// operations but, unlike __syncthreads, not for its global loads and stores -- loads that were
// issued early on purpose stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Workgroup inclusive scan; `wsum` is LDS with at least blockDim.x/64 + 1 words.  Returns the
// inclusive prefix of v for this thread and the workgroup total in *total.  Ends with a barrier,
// so wsum may be reused right after.  LDS_ONLY: its barriers are lds_barrier.
template <bool LDS_ONLY = false>
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wsum, uint32_t* total) {
    const int nw = blockDim.x >> 6;
    uint32_t incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) wsum[wave_id()] = incl;
    if constexpr (LDS_ONLY) lds_barrier(); else __syncthreads();
    // every wave scans the (at most 64) wave totals itself, lane l taking wsum[l]: one LDS read
    // and a DPP scan instead of a serial loop of dependent LDS reads
    const uint32_t x = (lane_id() < nw) ? wsum[lane_id()] : 0u;
    const uint32_t sc = wave_incl_scan(x);
    const int wv = __builtin_amdgcn_readfirstlane(wave_id());
    const uint32_t base = wv ? wave_read_lane(sc, wv - 1) : 0u;
    const uint32_t tot = wave_read_lane(sc, nw - 1);
    if constexpr (LDS_ONLY) lds_barrier(); else __syncthreads();
    *total = tot;
    return incl + base;
}

}  // namespace lshbeam
