// Log-softmax over the candidate list (Eq. 1 restricted to V_LSH) and beam expansion, on the
// device.  The paper copies P[B,|V|] to the host and heap-sorts there; here ONE workgroup per
// sentence finishes the softmax and selects the sentence's B best (beam, word) pairs directly
// over all B x C scores -- no per-row lists, no merge, nothing crosses workgroups.
//
//   1. Each wave takes hidden rows of the sentence.  The logits kernel left, per row and per
//      16-candidate tile, the pair (max logit, sum exp(logit - max)).  A row's log-sum-exp is
//      combined from those pairs, so no exponential is taken per logit here -- and the tile
//      maxima are all this kernel needs to read of most of the logits:
//   2. score = beam_score + (logit - lse).  Every lane keeps the best tile-maximum score it
//      strides over; the B-th largest of lane values (per wave by ranking for up to 16 beams,
//      over the whole workgroup by an LDS radix histogram for more) is a lower bound tau on the
//      B-th largest score overall, because B distinct scores (the maxima of B different tiles)
//      are >= tau.
//   3. Only tiles whose maximum reaches tau can hold a winner: they are listed workgroup-wide,
//      their 16 logits are read by the whole workgroup, and the scores >= tau -- a few B on
//      unordered data -- are appended to a short LDS list, which is ranked by counting: that
//      sorts it and the first B are the answer.
//   4. If the list overflows (heavily tied scores, or fewer tiles than beams) an exact 8-bit
//      radix select over all scores takes over.
//
// Selection works on 64-bit keys that are distinct by construction:
//   high 32 bits: order-preserving image of the fp32 score; low 32 bits: ~(beam << 24 | column),
// so "larger key" = "higher score, then lower beam, then lower column (= lower word id, the
// candidate list is ascending)", and the B-th key is unique.
#pragma once
#include <type_traits>
#include "device_utils.h"
#include "logits.h"

namespace lshbeam {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelListCap = 4096;    // short list of keys >= tau
constexpr int kSelRankCap = 1024;    // keys ranked directly (== kSelThreads)
constexpr int kSelRefineAbove = 256; // longer lists are thinned once more before ranking
constexpr int kSelBatch = 8;         // tile partials per lane and batch (a batch = 512 tiles of a row)
constexpr int kSelKeep = 4;          // batches of tile maxima a wave keeps in registers for pass 2
constexpr int kSelOpenCap = 4096;    // tiles whose maximum reaches tau (more: exact radix select)

__device__ __forceinline__ uint64_t make_key(float v, uint32_t index) {
    return ((uint64_t)f32_sortable(v + 0.0f) << 32) | (uint64_t)(~index);
}
__device__ __forceinline__ float key_value(uint64_t k) { return sortable_f32((uint32_t)(k >> 32)); }
__device__ __forceinline__ uint32_t key_index(uint64_t k) { return ~(uint32_t)k; }

// The k-th largest, k in 1..16, of the 64 lanes' values, all 32 bits resolved (scores accumulate
// over the steps of a sentence, and at |score| ~ 300 the low 12 bits of an fp32 span 0.1 -- a
// threshold that coarse would let thousands of scores through).  A sorting network on the DPP
// lane-permute paths: (1) every row of 16 lanes is sorted descending by a bitonic sort whose
// merges start with a mirror (partner = lane ^ (block - 1)), so that every compare-exchange
// points the same way and every partner pattern but "lane ^ 4" is one DPP modifier; (2) two
// sorted rows A, B are merged into the 16 largest of both by max(A[i], B[15 - i]) -- a bitonic
// sequence, sorted by four more butterfly stages -- first rows 0|1 and 2|3, then the two halves
// of the wave (these two exchanges cross rows and go through the LDS crossbar).  Every row ends
// up holding the wave's 16 largest in descending lane order.  ~90 vector instructions, against
// ~320 for ranking every lane against every other and ~10 dependent scalar instructions per bit
// for a bitwise descent on ballots.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_lane_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t dpp_lane_xor4(uint32_t x) {
    // lanes 0-3, 8-11 of a row read four lanes up (row_shl:4), the others four lanes down
    const int t = __builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xf, 0x5, false);
    return (uint32_t)__builtin_amdgcn_update_dpp(t, (int)x, 0x114, 0xf, 0xa, false);
}
__device__ __forceinline__ uint32_t keep_max_if(bool upper, uint32_t x, uint32_t p) {
    return upper ? max(x, p) : min(x, p);
}
__device__ __forceinline__ uint32_t wave_kth_largest_sort(uint32_t v, int k) {
    const int ln = lane_id();
    const bool b1 = (ln & 1) == 0, b2 = (ln & 2) == 0, b4 = (ln & 4) == 0, b8 = (ln & 8) == 0;
    constexpr int kXor1 = 0xB1, kXor2 = 0x4E, kXor3 = 0x1B;       // quad_perm
    constexpr int kXor7 = 0x141, kXor15 = 0x140, kXor8 = 0x128;   // half mirror, mirror, row_ror:8
    uint32_t x = v;
    x = keep_max_if(b1, x, dpp_lane_u32<kXor1>(x));
    x = keep_max_if(b2, x, dpp_lane_u32<kXor3>(x));
    x = keep_max_if(b1, x, dpp_lane_u32<kXor1>(x));
    x = keep_max_if(b4, x, dpp_lane_u32<kXor7>(x));
    x = keep_max_if(b2, x, dpp_lane_u32<kXor2>(x));
    x = keep_max_if(b1, x, dpp_lane_u32<kXor1>(x));
    x = keep_max_if(b8, x, dpp_lane_u32<kXor15>(x));
    x = keep_max_if(b4, x, dpp_lane_xor4(x));
    x = keep_max_if(b2, x, dpp_lane_u32<kXor2>(x));
    x = keep_max_if(b1, x, dpp_lane_u32<kXor1>(x));
#pragma unroll
    for (int cross = 0; cross < 2; ++cross) {
        // partner row, mirrored: lane ^ 31 pairs rows 0|1 and 2|3, lane ^ 47 rows 0|2 and 1|3
        const int partner = ln ^ (cross == 0 ? 31 : 47);
        x = max(x, (uint32_t)__builtin_amdgcn_ds_bpermute(partner << 2, (int)x));
        x = keep_max_if(b8, x, dpp_lane_u32<kXor8>(x));
        x = keep_max_if(b4, x, dpp_lane_xor4(x));
        x = keep_max_if(b2, x, dpp_lane_u32<kXor2>(x));
        x = keep_max_if(b1, x, dpp_lane_u32<kXor1>(x));
    }
    return wave_read_lane(x, k - 1);
}

// One wave's LDS operations complete in program order; this only keeps the compiler from moving
// them across the point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

struct SelShared {
    uint32_t open_list[kSelOpenCap];  // tiles to open: row << 20 | tile (tile < 2^20 as V <= 2^24)
    uint64_t list[kSelListCap];
    uint32_t rank[kSelRankCap];
    uint32_t hist[256];
    float lse[256];
    float bs[256];
    uint32_t wtau[kSelWaves];
    uint32_t misc[8];
};

// A lower bound tau of the k-th largest of the workgroup's 1024 thread values (k in 1..1024)
// that at least k and at most k + kSelSlack values reach (more only if more than that are equal
// in all resolved digits): radix descent, 8 bits per pass, on an LDS histogram.  A pass: clear
// the 256 bins, every thread still matching the resolved prefix adds itself to its digit's bin
// (a wave whose active lanes all share the digit -- the rule in the top byte -- adds once),
// wave 0 walks the bins from the top until the count crosses what is still needed.  It stops
// as soon as taking the whole crossing bin costs at most kSelSlack extra values; tau is that
// bin's lower edge.  Three barriers per pass and at most four passes, against one barrier per
// bit for a bitwise descent.
constexpr uint32_t kSelSlack = 8;
__device__ __forceinline__ uint32_t block_kth_largest_lb(uint32_t v, int k, SelShared* sh) {
    const int tid = threadIdx.x, ln = lane_id();
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) sh->hist[tid] = 0;
        __syncthreads();
        const bool act = (v & mask) == prefix;
        const uint32_t digit = (v >> shift) & 255u;
        const uint64_t actm = __ballot(act);
        if (actm) {
            const int first = __ffsll((unsigned long long)actm) - 1;
            const uint32_t d0 = wave_read_lane(digit, first);
            if (__ballot(act && digit == d0) == actm) {
                if (ln == first) atomicAdd(&sh->hist[d0], (uint32_t)__popcll(actm));
            } else if (act) {
                atomicAdd(&sh->hist[digit], 1u);
            }
        }
        __syncthreads();
        if (tid < kWave) {
            // lane L owns bins 255-4L .. 252-4L (descending): a scan over lanes walks the
            // histogram from the largest digit down; one lane sees the count cross `remaining`
            const int b0 = 255 - 4 * tid;
            uint32_t h[4], local = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { h[q] = sh->hist[b0 - q]; local += h[q]; }
            uint32_t excl = wave_incl_scan(local) - local;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (excl < remaining && remaining <= excl + h[q]) {
                    sh->misc[0] = (uint32_t)(b0 - q);
                    sh->misc[1] = remaining - excl;
                    sh->misc[2] = h[q];
                }
                excl += h[q];
            }
        }
        __syncthreads();
        const uint32_t bin = sh->misc[0], cnt = sh->misc[2];
        remaining = sh->misc[1];
        prefix |= bin << shift;
        mask |= 0xFFu << shift;
        if (cnt <= remaining + kSelSlack) break;
    }
    return prefix;
}

// Everything a sweep over the sentence's scores needs.
struct ScoreSrc {
    const float* logits;  // first row of the sentence
    int64_t cpitch;
    int B, C;
    const float* lse;     // LDS [B]
    const float* bs;      // LDS [B]
    __device__ __forceinline__ uint64_t key(int i, int c) const {
        const float score = bs[i] + (logits[(size_t)i * cpitch + c] - lse[i]);
        return make_key(score, ((uint32_t)i << 24) | (uint32_t)c);
    }
};

// Exact B largest keys by the whole workgroup: radix select, 8-bit digits, most significant
// first.  Writes them to list[] in any order.  Needs B*C > B.  Out of line: it only runs when
// more than kSelRankCap scores are left after thinning (heavy ties).
__device__ __noinline__ void block_radix_select(ScoreSrc src, int k, SelShared* sh) {
    // arguments of an out-of-line call arrive in vector registers: mark the uniform ones
    src.B = __builtin_amdgcn_readfirstlane(src.B);
    src.C = __builtin_amdgcn_readfirstlane(src.C);
    k = __builtin_amdgcn_readfirstlane(k);
    const int tid = threadIdx.x;
    uint64_t prefix = 0, mask = 0;
    uint32_t remaining = (uint32_t)k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) sh->hist[tid] = 0;
        __syncthreads();
        for (int i = 0; i < src.B; ++i)
            for (int c = tid; c < src.C; c += kSelThreads) {
                const uint64_t kk = src.key(i, c);
                if ((kk & mask) == prefix) atomicAdd(&sh->hist[(uint32_t)(kk >> shift) & 255u], 1u);
            }
        __syncthreads();
        if (tid < kWave) {
            // lane L owns bins 255-4L .. 252-4L (descending): a scan over lanes walks the
            // histogram from the largest digit down; one lane sees the count cross `remaining`
            const int b0 = 255 - 4 * tid;
            uint32_t h[4], local = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { h[q] = sh->hist[b0 - q]; local += h[q]; }
            uint32_t excl = wave_incl_scan(local) - local;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (excl < remaining && remaining <= excl + h[q]) {
                    sh->misc[0] = (uint32_t)(b0 - q);
                    sh->misc[1] = remaining - excl;
                    sh->misc[2] = h[q];
                }
                excl += h[q];
            }
        }
        __syncthreads();
        const uint32_t bin = sh->misc[0], cnt = sh->misc[2];
        remaining = sh->misc[1];
        prefix |= (uint64_t)bin << shift;
        mask |= 0xFFull << shift;
        if (cnt == remaining) break;  // the whole bin is taken: no need to refine further
    }
    if (tid == 0) sh->misc[3] = 0;
    __syncthreads();
    for (int i = 0; i < src.B; ++i)
        for (int c = tid; c < src.C; c += kSelThreads) {
            const uint64_t kk = src.key(i, c);
            if ((kk & mask) >= prefix) {
                const uint32_t pos = atomicAdd(&sh->misc[3], 1u);
                if (pos < (uint32_t)k) sh->list[pos] = kk;
            }
        }
    __syncthreads();
}

// Candidates per tile of the fused kernels: 16, the width of the matrix instruction, unless
// forced narrower (option fused_tile, 1..16; the unused columns of the instruction then idle).
// Measured on the 2224-candidate lists of the paper shape: 248 tiles of 9 on 256 workgroups, one
// each, are no faster than 139 tiles of 16 -- while the candidate rows arrive the machine as a
// whole is moving ~3.5 TB/s of scattered 4 KB rows, so it is the memory system, not the single CU,
// that sets those 2.5 us, and more tiles mean more records for the selection (+0.5 us).  The
// number of tiles never exceeds the record pitch.  Both the kernel that writes the records and
// the selection that reads them evaluate this rule.
constexpr int kMaxFusedGrid = 1024;   // workgroups per sentence at most
__host__ __device__ inline int select_tile_width(int C, int forced, int64_t ppitch) {
    int w = (forced > 0 && forced < 16) ? forced : 16;
    if (w < 16 && ((int64_t)C + w - 1) / w > ppitch) w = 16;
    return w;
}

// What the contraction kernels leave per (hidden row, tile): the fused kernels a TileRecord =
// float4 (max, sum exp, second largest, id of the max) and, in a parallel array, the second's id
// ("rich" records); the others the float2 (max, sum exp) alone.
template <typename REC> __device__ __forceinline__ REC empty_record();
template <> __device__ __forceinline__ float2 empty_record<float2>() { return make_float2(-INFINITY, 0.f); }
template <> __device__ __forceinline__ float4 empty_record<float4>() {
    return make_float4(-INFINITY, 0.f, -INFINITY, __int_as_float(-1));
}

// Loads of tile records / second ids.  SAME_KERNEL: the data was written by other workgroups of
// the running kernel (device-scope stores, store_shared_result), so it is read with device-scope
// loads, which do not hit in this XCD's caches -- cheaper than invalidating them (1.6 us measured
// for the fence against nothing for the loads, which miss anyway).
template <bool SAME_KERNEL>
__device__ __forceinline__ float2 load_record(const float2* p) { return *p; }
template <bool SAME_KERNEL>
__device__ __forceinline__ float4 load_record(const float4* p) {
    if constexpr (SAME_KERNEL) {
        const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
        const unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return make_float4(__uint_as_float((uint32_t)a), __uint_as_float((uint32_t)(a >> 32)),
                           __uint_as_float((uint32_t)b), __uint_as_float((uint32_t)(b >> 32)));
    } else {
        return *p;
    }
}
template <bool SAME_KERNEL>
__device__ __forceinline__ int32_t load_id2(const int32_t* p) {
    if constexpr (SAME_KERNEL) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}

// The first half of the selection for such records and a sentence of at most 64 beams: 16 lanes
// per hidden row, all rows at once, lane c of a row's sixteen taking records c, c + 16, ...  (A
// wave per row, as in the general path, spends a microsecond of instruction issue per row on a
// few dozen records.)  Leaves the rows' log-sum-exps and beam scores in LDS, lists every tile of
// every group whose maximum reaches tau in sh.open_list (count in sh.misc[5], which the caller
// has cleared) and returns tau.
__device__ __forceinline__ uint32_t select_front_grouped(SelShared& sh, int s, const float2* records, int64_t ppitch,
                                                         int ntiles, int G, int B, const float* beam_scores,
                                                         float* lse_out) {
    const int tid = threadIdx.x, ln = lane_id();
    const int row = tid >> 4, c = ln & 15;
    const bool row_ok = row < B;
    const float bsi = row_ok ? beam_scores[s * B + row] : 0.f;
    const float2* pr = records + ((size_t)s * B + min(row, B - 1)) * ppitch;
    const int nrec = group_records(ntiles, G);
    // Workgroup w of the G has ntiles / G tiles, one more if w < ntiles % G; record j is group
    // j / G of workgroup j % G.  While every workgroup has one group (the usual case) that is
    // group 0 of workgroup j: the divisions are taken only otherwise (a lane pays ~40
    // instructions for each, 16 waves sharing the CU's issue slots).
    const int full = ntiles / G, rem = ntiles - full * G;   // (uniform)
    const bool single = nrec <= G;
    // tiles of record j = group grp of workgroup w (0: a slot nobody wrote), and the first of them
    auto tiles_of_group = [&](int j, int w, int grp, int* first) {
        *first = w + kGroupTiles * grp * G;
        return j < nrec ? max(0, min(kGroupTiles, full + (w < rem ? 1 : 0) - kGroupTiles * grp)) : 0;
    };
    auto tiles_of = [&](int j, int* first) {
        return tiles_of_group(j, single ? j : j % G, single ? 0 : j / G, first);
    };
    // the records past the first 64 of a row, c + 64, c + 80, ...: (w, grp) kept up without dividing
    struct Walk { int j, w, grp; };
    auto walk_begin = [&]() {
        const int j = c + 16 * 4;
        return Walk{j, single ? j : j % G, single ? 0 : j / G};
    };
    auto walk_next = [&](Walk& it) {
        it.j += 16; it.w += 16;
        while (it.w >= G) { it.w -= G; ++it.grp; }
    };
    auto load = [&](int j, int n) {
        const float2 r = pr[min(j, max(nrec - 1, 0))];
        return n > 0 ? r : make_float2(-INFINITY, 0.f);
    };
    constexpr int KEPT = 4;                       // records per lane held in registers (64 per row)
    float2 r[KEPT];
    int ft[KEPT], nt[KEPT];
#pragma unroll
    for (int u = 0; u < KEPT; ++u) { nt[u] = tiles_of(c + 16 * u, &ft[u]); r[u] = load(c + 16 * u, nt[u]); }
    float m = fmaxf(fmaxf(r[0].x, r[1].x), fmaxf(r[2].x, r[3].x));
    if (nrec > 16 * KEPT) for (Walk it = walk_begin(); it.j < nrec; walk_next(it)) {
        int f;
        m = fmaxf(m, load(it.j, tiles_of_group(it.j, it.w, it.grp, &f)).x);
    }
    const float M = row16_max(m);
    float sum = 0.f;
    if (M != -INFINITY) {
#pragma unroll
        for (int u = 0; u < KEPT; ++u) sum += r[u].y * __expf(r[u].x - M);   // padding: 0 * 0
        if (nrec > 16 * KEPT) for (Walk it = walk_begin(); it.j < nrec; walk_next(it)) {
            int f;
            const float2 e = load(it.j, tiles_of_group(it.j, it.w, it.grp, &f));
            sum += e.y * __expf(e.x - M);
        }
    }
    const float lse = M + logf(row16_sum(sum));
    if (c == 0 && row_ok) { sh.lse[row] = lse; sh.bs[row] = bsi; lse_out[s * B + row] = lse; }
    const uint32_t lmax = (row_ok && m != -INFINITY) ? f32_sortable(bsi + (m - lse) + 0.0f) : 0u;
    const uint32_t tau = block_kth_largest_lb(lmax, B, &sh);
    // every tile of every group whose maximum reaches tau: one reservation per lane
    auto reaches = [&](float x) { return row_ok && x != -INFINITY && f32_sortable(bsi + (x - lse) + 0.0f) >= tau; };
    // Every instruction here is issued by all 16 waves, four to a SIMD, whether its lanes have
    // anything to list or not: one reservation per wave (the lanes' counts scanned on the DPP
    // network), and a wave skips the records none of its lanes lists.  A lane writes the (at most
    // eight) tiles of its record without a loop: the counts differ from lane to lane.
    auto put = [&](uint32_t pos, int first, int n) {
#pragma unroll
        for (int k = 0; k < kGroupTiles; ++k)
            if (k < n && pos + (uint32_t)k < (uint32_t)kSelOpenCap)
                sh.open_list[pos + k] = ((uint32_t)row << 20) | (uint32_t)(first + k * G);
    };
    int total = 0;
#pragma unroll
    for (int u = 0; u < KEPT; ++u) { if (!reaches(r[u].x)) nt[u] = 0; total += nt[u]; }
    {
        const uint32_t incl = wave_incl_scan((uint32_t)total);
        const uint32_t wave_total = wave_read_lane(incl, kWave - 1);
        if (wave_total) {   // (uniform)
            uint32_t base = 0;
            if (ln == 0) base = atomicAdd(&sh.misc[5], wave_total);
            uint32_t pos = wave_read_lane(base, 0) + incl - (uint32_t)total;   // this lane's first entry
#pragma unroll
            for (int u = 0; u < KEPT; ++u) {
                if (__ballot(nt[u] > 0) != 0ull) put(pos, ft[u], nt[u]);   // (uniform)
                pos += (uint32_t)nt[u];
            }
        }
    }
    if (nrec > 16 * KEPT) for (Walk it = walk_begin(); it.j < nrec; walk_next(it)) {
        int f;
        const int n = tiles_of_group(it.j, it.w, it.grp, &f);
        if (n > 0 && reaches(load(it.j, n).x)) {
            const uint32_t pos = atomicAdd(&sh.misc[5], (uint32_t)n);
            for (int k = 0; k < n; ++k)
                if (pos + (uint32_t)k < (uint32_t)kSelOpenCap) sh.open_list[pos + k] = ((uint32_t)row << 20) | (uint32_t)(f + k * G);
        }
    }
    return tau;
}

// The whole selection for the shape the fused kernels usually serve -- rich records, at most 16
// beams (a wave per hidden row), at most 512 tiles (eight records per lane) -- written out on its
// own, because this kernel is bound by instruction issue as much as by its trips to memory: the
// 16 waves of the workgroup share four SIMDs, a wave's vector instruction takes a SIMD for four
// cycles, and the general code below spends two fifths of its instructions on cases that cannot
// occur here (several batches per row, several rows per wave, records kept for a second pass).
// Same arithmetic and the same keys as the general path's short cut; returns false, having
// written nothing final, when that path has to decide: more than 64 listed entries, or a second
// largest among the B best (a tile may hide a third).  C_known < 0: the list's length is count[s];
// *C_out receives it.  Four records per lane are asked for before that length is known; a list
// of up to 256 tiles -- a dozen beams over a few thousand candidates -- then runs the code for
// four (Q = 4), a longer one asks for the rest and runs the code for eight.  The word id of a tile's second largest logit is
// fetched only when that logit reaches the threshold (on the benchmark's chained steps: never).
constexpr int kSmallQ = 8;
template <bool SAME_KERNEL, int Q>
__device__ __forceinline__ bool select_rich_small_body(SelShared& sh, int s, float bsi, float4 (&rec)[kSmallQ],
                                                       const int32_t* ids2_row, int ntiles, int B, float* lse_out,
                                                       int32_t* out_beam, int32_t* out_word, float* out_score) {
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    const bool has_row = wv < B;
    if (tid == 0) { sh.misc[4] = 0; sh.misc[6] = 0; }

    // log-sum-exp of the row, the lane's best tile maximum
    // (the arithmetic of the general path, operation for operation: the plans agree bit for bit)
    uint32_t best = 0;
    float lse = 0.f;
    if (has_row) {
        float m = -INFINITY;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ln + q * kWave >= ntiles) rec[q] = empty_record<float4>();
            m = fmaxf(m, rec[q].x);
        }
        float sum = 0.f;
        if (m != -INFINITY) {
#pragma unroll
            for (int q = 0; q < Q; ++q) sum += rec[q].y * __expf(rec[q].x - m);   // padding: 0 * 0
        }
        const float M = wave_max_f32(m);
        const float part = wave_sum_f32((m == -INFINITY) ? 0.f : sum * __expf(m - M));
        lse = M + logf(part);
        if (ln == 0) lse_out[s * B + wv] = lse;
        if (m != -INFINITY) best = f32_sortable(bsi + (m - lse) + 0.0f);
    }
    // tau: the largest over the rows of "B-th largest lane value of the row" (B distinct tile
    // maxima are >= it)
    // (waves without a row skip the sorting network: their issue slots are the others')
    const uint32_t kth = has_row ? wave_kth_largest_sort(best, B) : 0u;
    LSH_TRACE_ANY(2, 1);
    if (ln == 0) sh.wtau[wv] = kth;
    __syncthreads();
    uint32_t tau = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) tau = max(tau, sh.wtau[w]);

    // every largest / second largest score >= tau, one list reservation per wave.  A second
    // largest can reach tau only where the tile's largest does (the score is monotone in the
    // logit), so it is looked at only there; and a wave skips what none of its lanes needs.
    if (has_row) {
        uint32_t key1[Q], key2[Q];
        int32_t id2[Q];
        uint32_t mine = 0;
        bool any2 = false;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            key1[q] = f32_sortable(bsi + (rec[q].x - lse) + 0.0f);
            const bool in = ln + q * kWave < ntiles;
            if (!(in && __float_as_int(rec[q].w) >= 0 && key1[q] >= tau)) key1[q] = 0;   // (real keys are > 0)
            key2[q] = 0;
            id2[q] = -1;
            if (__ballot(key1[q] != 0) != 0ull) {   // (uniform)
                key2[q] = f32_sortable(bsi + (rec[q].z - lse) + 0.0f);
                if (!(key1[q] != 0 && key2[q] >= tau)) key2[q] = 0;
                any2 = any2 || key2[q] != 0;
                mine += key1[q] ? 1u : 0u;
            }
        }
        const bool seconds = __ballot(any2) != 0ull;   // (uniform; rare)
        if (seconds) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (key2[q]) id2[q] = load_id2<SAME_KERNEL>(ids2_row + ln + q * kWave);
                if (id2[q] < 0) key2[q] = 0;
                mine += key2[q] ? 1u : 0u;
            }
        }
        if (__ballot(mine != 0) != 0ull) {   // (uniform)
            const uint32_t incl = wave_incl_scan(mine);
            const uint32_t wave_total = wave_read_lane(incl, kWave - 1);
            uint32_t base = 0;
            if (ln == 0) base = atomicAdd(&sh.misc[4], wave_total);
            uint32_t pos = wave_read_lane(base, 0) + incl - mine;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (__ballot(key1[q] != 0) == 0ull) continue;   // (uniform)
                if (key1[q]) {
                    if (pos < (uint32_t)kWave) {
                        sh.list[pos] = ((uint64_t)key1[q] << 32) |
                                       (uint64_t)(~(((uint32_t)wv << 24) | (uint32_t)__float_as_int(rec[q].w)));
                        sh.open_list[pos] = 0u;
                    }
                    ++pos;
                }
                if (seconds && key2[q]) {
                    if (pos < (uint32_t)kWave) {
                        sh.list[pos] = ((uint64_t)key2[q] << 32) | (uint64_t)(~(((uint32_t)wv << 24) | (uint32_t)id2[q]));
                        sh.open_list[pos] = 1u;   // a second largest
                    }
                    ++pos;
                }
            }
        }
    }
    __syncthreads();
    const int mr = (int)sh.misc[4];
    LSH_TRACE_ANY(2, 3);
    if (mr > kWave) return false;   // (uniform; a longer list is the general path's)

    // ranks by ballot: in every wave lane j holds entry j, wave w ranks entries 4w .. 4w + 3
    const size_t o0 = (size_t)s * B;
    const uint64_t mine = (ln < mr) ? sh.list[ln] : 0ull;
    const uint32_t second = (ln < mr && sh.open_list[ln] != 0u) ? 1u : 0u;
    const uint32_t lo = (uint32_t)mine, hi = (uint32_t)(mine >> 32);
    uint64_t key = 0;
    uint32_t rank = 0xFFFFFFFFu, sec = 0;
#pragma unroll
    for (int q = 0; q < kWave / kSelWaves; ++q) {
        const int e = wv * (kWave / kSelWaves) + q;   // (wave-uniform)
        if (e >= mr) break;
        const uint64_t ke = ((uint64_t)wave_read_lane(hi, e) << 32) | wave_read_lane(lo, e);
        const uint32_t r = (uint32_t)__popcll(__ballot(mine > ke));
        const uint32_t se = wave_read_lane(second, e);
        if (ln == q) { key = ke; rank = r; sec = se; }
    }
    if (rank < (uint32_t)B) {   // (lanes 0..3 at most)
        if (sec) sh.misc[6] = 1u;
        const size_t o = o0 + rank;
        const float score = key_value(key);
        const uint32_t idx = key_index(key);
        const bool none = score == -INFINITY || score != score;
        out_beam[o] = none ? -1 : (int)(idx >> 24);
        out_word[o] = none ? -1 : (int)(idx & 0xFFFFFFu);
        out_score[o] = none ? -INFINITY : score;
    }
    if (wv == 0)
        for (int e = ln + min(mr, B); e < B; e += kWave) {
            out_beam[o0 + e] = -1; out_word[o0 + e] = -1; out_score[o0 + e] = -INFINITY;
        }
    LSH_TRACE_ANY(2, 4);
    __syncthreads();
    LSH_TRACE_ANY(2, 5);
    return sh.misc[6] == 0u;
}

template <bool SAME_KERNEL>
__device__ __forceinline__ bool select_rich_small(SelShared& sh, int s, const TileRecord* records, const int32_t* ids2,
                                                  int64_t ppitch, const int32_t* count, int C_known, int V, int B,
                                                  const float* beam_scores, float* lse_out, int32_t* out_beam,
                                                  int32_t* out_word, float* out_score, int tile_forced, int* C_out) {
    const int ln = lane_id(), wv = wave_id();
    LSH_TRACE_ANY(2, 0);
    // what is asked for at once, before the list's length is known: the row's beam score, its
    // first four records per lane (indices clamped to the allocated pitch; what lies past the
    // last tile is masked later) and the length.  A longer list's further records are asked for
    // when the length is here -- as many as it needs: every record loaded in vain costs this one
    // CU as much of its load rate as a real one (eight per lane up front: 0.3 us more on the
    // 139-tile list of the paper shape).
    float bsi = 0.f;
    float4 rec[kSmallQ];
    const size_t r0 = ((size_t)s * B + min(wv, B - 1)) * ppitch;
    if (wv < B) {
        bsi = beam_scores[s * B + wv];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            rec[q] = load_record<SAME_KERNEL>(records + r0 + min((int64_t)(ln + q * kWave), ppitch - 1));
    }
    const int C = C_known >= 0 ? C_known : (count ? count[s] : V);
    const int tn = select_tile_width(C, tile_forced, ppitch);
    const int ntiles = (C + tn - 1) / tn;
    *C_out = C;
    if (ntiles == 0 || ntiles > kSmallQ * kWave) return false;   // (uniform, like every return here)
    if (ntiles <= 4 * kWave)
        return select_rich_small_body<SAME_KERNEL, 4>(sh, s, bsi, rec, ids2 + r0, ntiles, B, lse_out, out_beam, out_word,
                                                      out_score);
#pragma unroll
    for (int q = 4; q < kSmallQ; ++q) {
        rec[q] = empty_record<float4>();
        if (wv < B && q * kWave < ntiles)   // (uniform)
            rec[q] = load_record<SAME_KERNEL>(records + r0 + min((int64_t)(ln + q * kWave), ppitch - 1));
    }
    return select_rich_small_body<SAME_KERNEL, 8>(sh, s, bsi, rec, ids2 + r0, ntiles, B, lse_out, out_beam, out_word,
                                                  out_score);
}

template <bool RICH, bool SAME_KERNEL = false, bool GROUPS = false>
__device__ __forceinline__ void select_sentence(SelShared& sh, int s, const float* logits, int64_t cpitch,
                                                const TileRecord* records, const int32_t* ids2, int64_t ppitch,
                                                const int32_t* cand, const int32_t* count, int C_known,
                                                int V, int B, const float* beam_scores, float* lse_out,
                                                int32_t* out_beam, int32_t* out_word, float* out_score,
                                                int tile_forced = 0, int rec_groups = 0) {
    if constexpr (RICH) {
        if (B <= kSelWaves) {
            int C_seen = C_known;
            if (select_rich_small<SAME_KERNEL>(sh, s, records, ids2, ppitch, count, C_known, V, B, beam_scores, lse_out,
                                               out_beam, out_word, out_score, tile_forced, &C_seen))
                return;
            C_known = C_seen;   // (the general path need not ask again)
            __syncthreads();    // (not this shape, or a tile may hide a winner: everybody has read the verdict)
        }
    }
    typedef typename std::conditional<RICH, float4, float2>::type REC;
    const REC* partials = reinterpret_cast<const REC*>(records);
    // batches of tile maxima a wave keeps in registers between the passes (rich records: also the
    // second largest and both ids, so one batch only)
    constexpr int KEEP = RICH ? 1 : kSelKeep;
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    LSH_TRACE_ANY(2, 0);
    // The first batch of records of this wave's first row is requested before the candidate
    // count is known (one memory round trip less): indices are clamped to the row's pitch, which
    // is allocated, and what lies beyond the last tile is masked after the load like any padding.
    // Lane r of a wave asks for the beam score of the wave's r-th row right away too: loads
    // return in order, so a score asked for inside the loop over the rows would have every
    // iteration wait for a memory round trip (and for the records requested ahead of it).
    float bs_pre = 0.f;
    constexpr bool grouped = GROUPS;
    if (!grouped && wv + ln * kSelWaves < B) bs_pre = beam_scores[s * B + wv + ln * kSelWaves];   // (B <= 256: ln < 16)
    REC first_batch[kSelBatch];
    int32_t first_ids2[kSelBatch];
#pragma unroll
    for (int q = 0; q < kSelBatch; ++q) { first_batch[q] = empty_record<REC>(); first_ids2[q] = -1; }
    if (wv < B && !grouped) {
        const size_t r0 = ((size_t)s * B + wv) * ppitch;
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q) {
            const int64_t at = min((int64_t)(ln + q * kWave), ppitch - 1);
            first_batch[q] = load_record<SAME_KERNEL>(partials + r0 + at);
            if constexpr (RICH && KEEP > 0) first_ids2[q] = load_id2<SAME_KERNEL>(ids2 + r0 + at);
        }
    }
    const int C = C_known >= 0 ? C_known : (count ? count[s] : V);
    // candidates per tile: 16, or what the fused kernel that wrote the records was told to use
    const int tn = RICH ? select_tile_width(C, tile_forced, ppitch) : 16;
    const int ntiles = (C + tn - 1) / tn;
    // GROUPS: the records stand for groups of tiles (select_front_grouped; rec_groups = the
    // workgroups per sentence of the kernel that wrote them; at most 64 beams)
    static_assert(!(GROUPS && RICH), "rich records are per tile");
    const int nrec = ntiles;
    const float* lg = logits + (size_t)s * B * cpitch;
    if (tid == 0) { sh.misc[4] = 0; sh.misc[5] = 0; sh.misc[6] = 0; }
    // Ranks the m <= kSelRankCap keys of sh.list by counting (the inner loop split over the
    // workgroup: thread t compares key e = t % m with one of `parts` slices of the list); ends
    // with a barrier, ranks in sh.rank.
    auto rank_list = [&](int m) {
        if (tid < m) sh.rank[tid] = 0;
        __syncthreads();
        if (m > 0) {
            const int parts = kSelThreads / m;
            const int e = tid % m, p = tid / m;
            if (p < parts) {
                const int chunk = (m + parts - 1) / parts;
                const int j0 = p * chunk, j1 = min(m, j0 + chunk);
                const uint64_t mine = sh.list[e];
                uint32_t rank = 0;
#pragma unroll 8
                for (int j = j0; j < j1; ++j) rank += (sh.list[j] > mine) ? 1u : 0u;
                if (rank) atomicAdd(&sh.rank[e], rank);
            }
        }
        __syncthreads();
    };
    // Results from the ranked list: rank r < B goes to slot r; slots beyond the number of finite
    // scores are (-1, -1, -inf).  The low 24 bits of a key's index are a word id (ids_in_keys) or
    // a column of the candidate list.
    const size_t o0 = (size_t)s * B;
    auto emit = [&](int m, bool ids_in_keys) {
        for (int e = tid + min(m, B); e < B; e += kSelThreads) {
            out_beam[o0 + e] = -1; out_word[o0 + e] = -1; out_score[o0 + e] = -INFINITY;
        }
        if (tid < m && sh.rank[tid] < (uint32_t)B) {
            const uint64_t k = sh.list[tid];
            const size_t o = o0 + sh.rank[tid];
            const float score = key_value(k);
            const uint32_t idx = key_index(k);
            if (score == -INFINITY || score != score) {
                out_beam[o] = -1; out_word[o] = -1; out_score[o] = -INFINITY;
            } else {
                const int c = (int)(idx & 0xFFFFFFu);
                out_beam[o] = (int)(idx >> 24);
                out_word[o] = (ids_in_keys || !cand) ? c : cand[(size_t)s * V + c];
                out_score[o] = score;
            }
        }
    };

    const ScoreSrc src{lg, cpitch, B, C, sh.lse, sh.bs};
    uint32_t tau;
    if (grouped) {
        __syncthreads();   // (the counters)
        tau = select_front_grouped(sh, s, reinterpret_cast<const float2*>(records), ppitch, ntiles, rec_groups, B,
                                   beam_scores, lse_out);
        LSH_TRACE_ANY(2, 2);
    } else {   // (down to the second pass's list of tiles; not indented)

    // ---- per row: log-sum-exp from the tile records, and the lane's best tile-maximum score.
    //      Wave w takes rows w, w + 16, ...; a row is visited in batches of 512 tiles.  The
    //      records were written by other XCDs, so every load is a trip to memory: the next
    //      batch (of this row or of the wave's next row) is requested before the current one is
    //      reduced, and loads are never branched around (indices are clamped, padding is masked
    //      after the load). ----
    uint32_t lmax = 0;
    // The tile maxima of the wave's first KEEP batches stay in registers for the second pass
    // (rich records: also the second largest and both ids).
    constexpr int KR = KEEP > 0 ? KEEP : 1;
    float keep[KR][kSelBatch];
    float keep_z[RICH ? KR : 1][kSelBatch];
    int32_t keep_id1[RICH ? KR : 1][kSelBatch], keep_id2[RICH ? KR : 1][kSelBatch];
    constexpr int kBatchTiles = kWave * kSelBatch;
    const int nb = (nrec + kBatchTiles - 1) / kBatchTiles;                     // batches per row
    const int nit = (wv < B ? (B - wv + kSelWaves - 1) / kSelWaves : 0) * nb;    // of this wave
    // lanes x kSelBatch slots of a batch that hold tiles at all (wave-uniform; the rest is
    // skipped outright: 16 waves on one CU are bound by instruction issue)
    auto slots_of = [&](int bt) { return min(kSelBatch, (nrec - bt * kBatchTiles + kWave - 1) / kWave); };
    auto load_batch = [&](int it, REC (&p)[kSelBatch]) {
        const int r = it / nb, bt = it - r * nb;
        const int nq = slots_of(bt);
        const REC* pr = partials + ((size_t)s * B + (wv + r * kSelWaves)) * ppitch;
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q)
            if (q < nq) p[q] = load_record<SAME_KERNEL>(pr + min(bt * kBatchTiles + ln + q * kWave, nrec - 1));
    };
    auto load_ids2 = [&](int it, int32_t (&p)[kSelBatch]) {
        const int r = it / nb, bt = it - r * nb;
        const int nq = slots_of(bt);
        const int32_t* pr = ids2 + ((size_t)s * B + (wv + r * kSelWaves)) * ppitch;
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q)
            if (q < nq) p[q] = load_id2<SAME_KERNEL>(pr + min(bt * kBatchTiles + ln + q * kWave, nrec - 1));
    };
    {
        REC cur[kSelBatch], nxt[kSelBatch];
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q) cur[q] = first_batch[q];
        float m = -INFINITY, sum = 0.f, lmx = -INFINITY, bsi = 0.f;
        for (int it = 0; it < nit; ++it) {
            const int r = it / nb, bt = it - r * nb;
            const int i = wv + r * kSelWaves;
            const int nq = slots_of(bt);
            if (it + 1 < nit) load_batch(it + 1, nxt);
            if (bt == 0) {
                m = -INFINITY; sum = 0.f; lmx = -INFINITY;
                bsi = __uint_as_float(wave_read_lane(__float_as_uint(bs_pre), r));
            }
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q)
                if (q >= nq || bt * kBatchTiles + ln + q * kWave >= nrec)
                    cur[q] = empty_record<REC>();
            if constexpr (KEEP > 0) {
#pragma unroll
                for (int k = 0; k < KEEP; ++k)  // registers cannot be indexed at run time
                    if (k == it) {
#pragma unroll
                        for (int q = 0; q < kSelBatch; ++q) {
                            keep[k][q] = cur[q].x;
                            if constexpr (RICH) {
                                keep_z[k][q] = cur[q].z;
                                keep_id1[k][q] = __float_as_int(cur[q].w);
                            }
                        }
                    }
            }
            float bm = cur[0].x;
#pragma unroll
            for (int q = 1; q < kSelBatch; ++q)
                if (q < nq) bm = fmaxf(bm, cur[q].x);
            lmx = fmaxf(lmx, bm);
            if (bm > m) { sum *= __expf(m - bm); m = bm; }
            if (m != -INFINITY) {
#pragma unroll
                for (int q = 0; q < kSelBatch; ++q)
                    if (q < nq) sum += cur[q].y * __expf(cur[q].x - m);  // padding: 0 * 0
            }
            if (bt == nb - 1) {
                const float M = wave_max_f32(m);
                const float part = wave_sum_f32((m == -INFINITY) ? 0.f : sum * __expf(m - M));
                const float lse = M + logf(part);
                if (ln == 0) { sh.lse[i] = lse; sh.bs[i] = bsi; lse_out[s * B + i] = lse; }
                if (lmx != -INFINITY) lmax = max(lmax, f32_sortable(bsi + (lmx - lse) + 0.0f));
            }
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) cur[q] = nxt[q];
        }
    }
    if constexpr (RICH && KEEP > 0) {
        // (only batch 0 of the wave's first row can be in first_ids2; KEEP is 1 for rich records)
        static_assert(KEEP == 1, "rich records keep one batch");
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q) keep_id2[0][q] = first_ids2[q];
    }
    if (nb == 0) {  // empty candidate list: every row's log-sum-exp is -inf
        for (int i = wv; i < B; i += kSelWaves)
            if (ln == 0) {
                sh.lse[i] = -INFINITY; sh.bs[i] = beam_scores[s * B + i]; lse_out[s * B + i] = -INFINITY;
            }
    }
    LSH_TRACE_ANY(2, 1);

    // ---- threshold tau: a lower bound of the B-th best score from the 16 x 64 lane values
    //      (B distinct tile maxima are >= it).  Up to 16 beams every row has its own wave, and
    //      the largest over the waves of "B-th largest lane value in the wave" costs no barrier
    //      per bit; with more beams the B-th largest of all 1024 lane values is much tighter. ----
    if (B <= kSelWaves) {
        const uint32_t kth = wave_kth_largest_sort(lmax, B);
        if (ln == 0) sh.wtau[wv] = kth;
        __syncthreads();
        tau = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) tau = max(tau, sh.wtau[w]);
    } else {
        tau = block_kth_largest_lb(lmax, B, &sh);
    }
    LSH_TRACE_ANY(2, 2);

    if constexpr (RICH) {
        // ---- the short cut: every largest / second largest score >= tau, from the records ----
        // (no barrier needed here: the counters were cleared before the barriers of the tau
        // computation, and a wave reads back only the lse / beam score of its own rows)
        wave_lds_sync();
        for (int it = 0; it < nit; ++it) {
            const int r = it / nb, bt = it - r * nb;
            const int i = wv + r * kSelWaves;
            const int t0 = bt * kBatchTiles;
            const float lse = sh.lse[i], bsi = sh.bs[i];
            float x1[kSelBatch], x2[kSelBatch];
            int32_t i1[kSelBatch], i2[kSelBatch];
            bool have = false;
            if constexpr (KEEP > 0) {
                if (it < KEEP) {
                    have = true;
#pragma unroll
                    for (int k = 0; k < KEEP; ++k)
                        if (k == it) {
#pragma unroll
                            for (int q = 0; q < kSelBatch; ++q) {
                                x1[q] = keep[k][q]; x2[q] = keep_z[k][q];
                                i1[q] = keep_id1[k][q]; i2[q] = keep_id2[k][q];
                            }
                        }
                }
            }
            if (!have) {
                REC p[kSelBatch];
#pragma unroll
                for (int q = 0; q < kSelBatch; ++q) { p[q] = empty_record<REC>(); i2[q] = -1; }
                load_batch(it, p);
                load_ids2(it, i2);
#pragma unroll
                for (int q = 0; q < kSelBatch; ++q) {
                    x1[q] = p[q].x; x2[q] = p[q].z; i1[q] = __float_as_int(p[q].w);
                }
            }
            const int nq = slots_of(bt);
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) {
                if (q >= nq) continue;  // wave-uniform
                const bool in = t0 + ln + q * kWave < nrec;
                const float s1 = bsi + (x1[q] - lse), s2 = bsi + (x2[q] - lse);
                if (in && i1[q] >= 0 && f32_sortable(s1 + 0.0f) >= tau) {
                    const uint32_t pos = atomicAdd(&sh.misc[4], 1u);
                    if (pos < (uint32_t)kSelListCap) {
                        sh.list[pos] = make_key(s1, ((uint32_t)i << 24) | (uint32_t)i1[q]);
                        sh.open_list[pos] = 0u;
                    }
                }
                if (in && i2[q] >= 0 && f32_sortable(s2 + 0.0f) >= tau) {
                    const uint32_t pos = atomicAdd(&sh.misc[4], 1u);
                    if (pos < (uint32_t)kSelListCap) {
                        sh.list[pos] = make_key(s2, ((uint32_t)i << 24) | (uint32_t)i2[q]);
                        sh.open_list[pos] = 1u;   // a second largest
                    }
                }
            }
        }
        __syncthreads();
        LSH_TRACE_ANY(2, 6);
        const int mr = (int)sh.misc[4];
        if (mr <= kWave) {
            // The usual case, a few dozen keys: in every wave lane j holds key j, and wave w ranks
            // keys 4w .. 4w + 3, each by one ballot ("which keys are larger?").  A key among the
            // B best is written out at once; if one of them is a second largest, the verdict word
            // sends everybody on to the general path, which writes all B results again.  (One
            // wave ranking all keys by a loop of lane broadcasts took 0.6 us; all 16 waves ranking
            // all keys, to save the barrier, was slower still: they share four instruction issuers.)
            {
                const uint64_t mine = (ln < mr) ? sh.list[ln] : 0ull;   // (real keys are never 0)
                const uint32_t second = (ln < mr && sh.open_list[ln] != 0u) ? 1u : 0u;
                const uint32_t lo = (uint32_t)mine, hi = (uint32_t)(mine >> 32);
                uint64_t key = 0;
                uint32_t rank = 0xFFFFFFFFu, sec = 0;
#pragma unroll
                for (int q = 0; q < kWave / kSelWaves; ++q) {
                    const int e = wv * (kWave / kSelWaves) + q;   // (wave-uniform)
                    if (e >= mr) break;
                    const uint64_t ke = ((uint64_t)wave_read_lane(hi, e) << 32) | wave_read_lane(lo, e);
                    const uint32_t r = (uint32_t)__popcll(__ballot(mine > ke));
                    const uint32_t se = wave_read_lane(second, e);
                    if (ln == q) { key = ke; rank = r; sec = se; }
                }
                if (rank < (uint32_t)B) {   // (lanes 0..3 at most)
                    if (sec) sh.misc[6] = 1u;
                    const size_t o = o0 + rank;
                    const float score = key_value(key);
                    const uint32_t idx = key_index(key);
                    const bool none = score == -INFINITY || score != score;
                    out_beam[o] = none ? -1 : (int)(idx >> 24);
                    out_word[o] = none ? -1 : (int)(idx & 0xFFFFFFu);
                    out_score[o] = none ? -INFINITY : score;
                }
                if (wv == 0)
                    for (int e = ln + min(mr, B); e < B; e += kWave) {
                        out_beam[o0 + e] = -1; out_word[o0 + e] = -1; out_score[o0 + e] = -INFINITY;
                    }
            }
            LSH_TRACE_ANY(2, 4);
            __syncthreads();
            if (sh.misc[6] == 0u) {
                LSH_TRACE_ANY(2, 5);
                return;
            }
        } else if (mr <= kSelRankCap) {   // (workgroup-uniform)
            rank_list(mr);
            if (tid < mr && sh.rank[tid] < (uint32_t)B && sh.open_list[tid]) sh.misc[6] = 1u;
            __syncthreads();
            if (sh.misc[6] == 0u) {
                LSH_TRACE_ANY(2, 4);
                emit(mr, true);
                LSH_TRACE_ANY(2, 5);
                return;
            }
        }
        __syncthreads();
        if (tid == 0) sh.misc[4] = 0;
        // (logits and candidate ids are read with plain loads below: none of them may come from
        // a cache line fetched before the other workgroups' stores)
        if constexpr (SAME_KERNEL) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        __syncthreads();
    }

    // ---- second pass: tiles whose maximum reaches tau are opened, 16 lanes per tile ----
    // (a) every wave lists the tiles of its rows that qualify in one workgroup-wide LDS list:
    //     which rows hold them is as uneven as the beam scores (the best beam's row can hold
    //     nearly all), so they are opened by the whole workgroup, not by the row's wave
    for (int it = 0; it < nit; ++it) {
        const int r = it / nb, bt = it - r * nb;
        const int i = wv + r * kSelWaves;
        const int t0 = bt * kBatchTiles;
        const float lse = sh.lse[i], bsi = sh.bs[i];
        float px[kSelBatch];  // the batch's tile maxima
        bool have = false;
        if constexpr (KEEP > 0) {
            if (it < KEEP) {
                have = true;
#pragma unroll
                for (int k = 0; k < KEEP; ++k)
                    if (k == it) {
#pragma unroll
                        for (int q = 0; q < kSelBatch; ++q) px[q] = keep[k][q];
                    }
            }
        }
        if (!have) {
            REC p[kSelBatch];
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) p[q] = empty_record<REC>();
            load_batch(it, p);
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) px[q] = p[q].x;
        }
        // most batches hold no qualifying tile: one test on the lane's best of the batch
        // settles that (bound by instruction issue, 16 waves on one CU)
        float best = px[0];
#pragma unroll
        for (int q = 1; q < kSelBatch; ++q) best = fmaxf(best, px[q]);
        if (__ballot(f32_sortable(bsi + (best - lse) + 0.0f) >= tau) == 0) continue;
        uint64_t bal[kSelBatch];
        uint32_t n_mine = 0;
        const int nq = slots_of(bt);  // slots of the batch that hold tiles at all (wave-uniform)
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q) {
            bal[q] = 0;
            if (q < nq) {
                const int t = t0 + ln + q * kWave;
                bal[q] = __ballot(t < nrec && f32_sortable(bsi + (px[q] - lse) + 0.0f) >= tau);
                n_mine += (uint32_t)__popcll(bal[q]);
            }
        }
        if (n_mine) {  // wave-uniform
            uint32_t base = 0;
            if (ln == 0) base = atomicAdd(&sh.misc[5], n_mine);
            base = wave_read_lane(base, 0);
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) {
                if (bal[q] == 0) continue;  // wave-uniform
                const uint32_t pos = base + lanes_below(bal[q]);
                if (((bal[q] >> ln) & 1ull) && pos < (uint32_t)kSelOpenCap)
                    sh.open_list[pos] = ((uint32_t)i << 20) | (uint32_t)(t0 + ln + q * kWave);
                base += (uint32_t)__popcll(bal[q]);
            }
        }
    }
    }   // (!grouped)
    LSH_TRACE_ANY(2, 6);
    __syncthreads();
    LSH_TRACE_ANY(2, 7);
    // (b) 16 lanes per tile, 64 tiles per sweep of the workgroup, four sweeps in flight -- eight
    //     when that makes one round trip to memory of two (the logits were written by other
    //     XCDs: every sweep batch is a cold read)
    const uint32_t n_open = sh.misc[5];
    if (n_open <= (uint32_t)kSelOpenCap) {
        auto open_tiles = [&](auto in_flight) {
            constexpr int U = decltype(in_flight)::value;
            for (uint32_t g0 = (uint32_t)(tid >> 4); g0 < n_open; g0 += U * (kSelThreads / 16)) {
                float x[U], lsev[U], bsq[U];
                int c[U], iq[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t j = g0 + u * (kSelThreads / 16);
                    const uint32_t ent = sh.open_list[min(j, n_open - 1)];
                    iq[u] = (int)(ent >> 20);
                    const int cc = (int)(ent & 0xFFFFFu) * tn + (ln & 15);
                    c[u] = (j < n_open && (ln & 15) < tn && cc < C) ? cc : -1;
                    x[u] = lg[(size_t)iq[u] * cpitch + max(c[u], 0)];
                    lsev[u] = sh.lse[iq[u]];
                    bsq[u] = sh.bs[iq[u]];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float sc = bsq[u] + (x[u] - lsev[u]);
                    if (c[u] >= 0 && f32_sortable(sc + 0.0f) >= tau) {
                        const uint32_t pos = atomicAdd(&sh.misc[4], 1u);
                        if (pos < (uint32_t)kSelListCap)
                            sh.list[pos] = make_key(sc, ((uint32_t)iq[u] << 24) | (uint32_t)c[u]);
                    }
                }
            }
        };
        if (n_open > 4u * (kSelThreads / 16) && n_open <= 8u * (kSelThreads / 16))
            open_tiles(std::integral_constant<int, 8>{});
        else
            open_tiles(std::integral_constant<int, 4>{});
        LSH_TRACE_ANY(2, 8);
    } else if (tid == 0) {
        sh.misc[4] = kSelListCap + 1;  // too many qualifying tiles (heavy ties): exact select below
    }
    __syncthreads();
    int m = (int)sh.misc[4];
    LSH_TRACE_ANY(2, 3);
#ifdef LSHBEAM_TRACE
    if (tid == 0) {
        g_trace[2][10] = g_trace[2][0] + n_open;  // counts, printed as offsets from slot 0
        g_trace[2][11] = g_trace[2][0] + (unsigned)m;
    }
#endif
    // A long list (many near-equal tile maxima, e.g. many beams) is thinned once more with the
    // same argument applied to the list itself: thread t owns keys t, t+1024, ...; the B-th
    // largest thread maximum bounds the B-th largest key from below.
    if (m > kSelRefineAbove && m <= kSelListCap && m > B) {
        uint64_t mine[kSelListCap / kSelThreads];
        uint32_t tm = 0;
#pragma unroll
        for (int q = 0; q < kSelListCap / kSelThreads; ++q) {
            const int e = tid + q * kSelThreads;
            mine[q] = (e < m) ? sh.list[e] : 0ull;
            tm = max(tm, (uint32_t)(mine[q] >> 32));
        }
        const uint32_t tau2 = block_kth_largest_lb(tm, B, &sh);  // m > 256 >= B keys exist
        if (tid == 0) sh.misc[4] = 0;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kSelListCap / kSelThreads; ++q) {
            if (tid + q * kSelThreads < m && (uint32_t)(mine[q] >> 32) >= tau2) {
                const uint32_t pos = atomicAdd(&sh.misc[4], 1u);
                sh.list[pos] = mine[q];  // pos < m <= kSelListCap; every old key is in registers
            }
        }
        __syncthreads();
        m = (int)sh.misc[4];
    }
    if (m > kSelRankCap) {
        __syncthreads();
        block_radix_select(src, B, &sh);
        m = B;
    }
    rank_list(m);
    LSH_TRACE_ANY(2, 4);
    emit(m, false);
    LSH_TRACE_ANY(2, 5);
}

// grid = S workgroups (one per sentence), kSelThreads threads: the selection as a kernel of its
// own, after kernels that left rich (fused plans) or plain tile records.
template <bool RICH, bool GROUPS>
__global__ void __launch_bounds__(kSelThreads)
k_select(const float* __restrict__ logits, int64_t cpitch, const TileRecord* __restrict__ records,
         const int32_t* __restrict__ ids2, int64_t ppitch, const int32_t* __restrict__ cand,
         const int32_t* __restrict__ count, int V, int B, const float* __restrict__ beam_scores,
         float* __restrict__ lse_out /*[R]*/, int32_t* __restrict__ out_beam,
         int32_t* __restrict__ out_word, float* __restrict__ out_score, int tile_forced, int rec_groups) {
    __shared__ SelShared sh;
    select_sentence<RICH, false, GROUPS>(sh, (int)blockIdx.x, logits, cpitch, records, ids2, ppitch, cand, count, -1,
                                         V, B, beam_scores, lse_out, out_beam, out_word, out_score, tile_forced,
                                         rec_groups);
}

// lp[i, c] = logit[i, c] - lse[i] for one sentence, for inspection.
__global__ void __launch_bounds__(256)
k_logprobs_dump(const float* __restrict__ logits, int64_t cpitch, const float* __restrict__ lse,
                int row0, int B, int C, float* __restrict__ out, int64_t opitch) {
    const int i = blockIdx.y;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B && c < C) out[(size_t)i * opitch + c] = logits[(size_t)(row0 + i) * cpitch + c] - lse[row0 + i];
}

}  // namespace lshbeam
