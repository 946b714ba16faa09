// Log-softmax over the candidate list (Eq. 1 restricted to V_LSH) and beam expansion, on the
// device.  The paper copies P[B,|V|] to the host and heap-sorts there; here one workgroup per
// hidden row reduces its logits to (log-sum-exp, its B best columns), and the last workgroup of
// a sentence to finish merges the B partial lists into the sentence's B best (beam, word) pairs.
//
// A row's B best raw logits are a superset of what that row can contribute to the sentence's
// top B (score = beam_score + logit - lse is increasing in logit inside a row), so selection on
// raw logits loses nothing.
//
// Selection works on 64-bit keys that are distinct by construction:
//   high 32 bits: order-preserving image of the fp32 value; low 32 bits: ~(tie-break index),
// so "larger key" means "larger value, then lower index" and the k-th key is unique.
//
// block_topk_sorted finds the k largest keys exactly in two sweeps over the data (the second
// sweep of a logit row hits the vector cache: a row of a few thousand floats was just read):
//   1. every thread takes the maximum of the keys it strides over; from those 256 thread maxima a
//      lower bound tau on the k-th largest key overall is derived (at least k distinct elements
//      are >= tau), so every winner is >= tau;
//   2. keys >= tau are appended to a short LDS list (a few k of them on unordered data) and
//      ranked against each other by counting, which also leaves them sorted.
// When all n keys fit the list, step 1 is skipped (tau = 0).
// If the list overflows (heavily tied data) an exact 8-bit radix select takes over.
#pragma once
#include "device_utils.h"

namespace lshbeam {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelListCap = 512;      // short list of keys >= tau
constexpr int kSelBatch = 8;          // independent loads in flight per thread in the row sweep
constexpr int kSelMergeLds = 4096;    // merge keys kept in LDS up to this many

struct SelScratch {  // LDS
    uint32_t hist[256];
    uint32_t tmax[kSelThreads];
    uint64_t list[kSelListCap];
    uint32_t sh[8];
    float redm[kSelWaves];
    float reds[kSelWaves];
};

__device__ __forceinline__ uint64_t make_key(float v, uint32_t index) {
    return ((uint64_t)f32_sortable(v + 0.0f) << 32) | (uint64_t)(~index);
}
__device__ __forceinline__ float key_value(uint64_t k) { return sortable_f32((uint32_t)(k >> 32)); }
__device__ __forceinline__ uint32_t key_index(uint64_t k) { return ~(uint32_t)k; }

// Where the n keys of a selection come from: a row of fp32 logits (key = value, column) or an
// array of ready-made keys.  Thread t owns elements t, t+256, ...
struct KeySrc {
    const float* row;
    const uint64_t* keys;
    int n;
    __device__ __forceinline__ uint64_t key(int i) const {
        return row ? make_key(row[i], (uint32_t)i) : keys[i];
    }
};

// Exact radix select (8-bit digits, most significant first) of the k largest of the n distinct
// keys; writes them to out[] in any order.  Requires n > k.  All threads must call it.  Kept out
// of line: it only runs when the short list of block_topk_sorted overflows.
__device__ __noinline__ void block_radix_select(KeySrc src, int k, uint64_t* out, SelScratch* sc) {
    const int tid = threadIdx.x;
    // arguments of an out-of-line call arrive in vector registers: tell the compiler the
    // workgroup-uniform ones are uniform
    src.n = __builtin_amdgcn_readfirstlane(src.n);
    k = __builtin_amdgcn_readfirstlane(k);
    uint64_t prefix = 0, mask = 0;
    uint32_t remaining = (uint32_t)k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        sc->hist[tid] = 0;  // kSelThreads == 256 bins
        __syncthreads();
        for (int i = tid; i < src.n; i += kSelThreads) {
            const uint64_t kk = src.key(i);
            if ((kk & mask) == prefix) atomicAdd(&sc->hist[(uint32_t)(kk >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            // lane L owns bins 255-4L .. 252-4L (descending), so a scan over lanes walks the
            // histogram from the largest digit down
            const int b0 = 255 - 4 * tid;
            uint32_t h[4], local = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { h[q] = sc->hist[b0 - q]; local += h[q]; }
            const uint32_t incl = wave_incl_scan(local);
            uint32_t excl = incl - local;
            if (excl < remaining && remaining <= incl) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (excl < remaining && remaining <= excl + h[q]) {
                        sc->sh[0] = (uint32_t)(b0 - q);
                        sc->sh[1] = remaining - excl;
                        sc->sh[2] = h[q];
                    }
                    excl += h[q];
                }
            }
        }
        __syncthreads();
        const uint32_t bin = sc->sh[0], cnt = sc->sh[2];
        remaining = sc->sh[1];
        prefix |= (uint64_t)bin << shift;
        mask |= 0xFFull << shift;
        if (cnt == remaining) break;  // the whole bin is taken: no need to refine further
    }
    if (tid == 0) sc->sh[3] = 0;
    __syncthreads();
    for (int i = tid; i < src.n; i += kSelThreads) {
        const uint64_t kk = src.key(i);
        if ((kk & mask) >= prefix) {
            const uint32_t pos = atomicAdd(&sc->sh[3], 1u);
            if (pos < (uint32_t)k) out[pos] = kk;
        }
    }
    __syncthreads();
}

// The k largest of the n distinct keys of `src`, written to out[] in DESCENDING order.
// `lmax32` is the maximum of the high key words over this thread's elements (0 if it owns none).
// Returns min(n, k).  `out` may be global or LDS; it is complete after the trailing barrier.
// All threads must call it.
__device__ __forceinline__ int block_topk_sorted(KeySrc src, int k, uint32_t lmax32, uint64_t* out,
                                                 SelScratch* sc) {
    const int tid = threadIdx.x, n = src.n;
    LSH_TRACE(2, 8);
    if (tid == 0) { sc->sh[3] = 0; sc->sh[5] = 0; }
    if (n > k && n > kSelListCap) {
        // A lower bound tau on the k-th largest key from the 256 thread maxima, without sorting
        // them: inside each wave the kw-th largest of its 64 lane maxima is found exactly by a
        // bitwise radix descent on wave ballots (no LDS, no barrier).
        //   k <= 64: kw = k, tau = the largest of the four wave results (that wave alone has k
        //            thread maxima, hence k distinct elements, >= tau);
        //   k  > 64: kw = ceil(k/4), tau = the smallest of the four (4*kw >= k elements >= tau).
        const int kw = (k <= kWave) ? k : (k + kSelWaves - 1) / kSelWaves;
        uint64_t active = ~0ull;   // all of this is wave-uniform and lives in scalar registers
        uint32_t kth = 0;
        int need = kw;
        // the low 12 mantissa bits are left at zero: still a lower bound, 12 fewer serial steps
#pragma unroll 4
        for (int bit = 31; bit >= 12; --bit) {
            const uint64_t ones = __ballot((lmax32 >> bit) & 1u) & active;
            const int c = __popcll(ones);
            if (c >= need) { active = ones; kth |= 1u << bit; }
            else { need -= c; active &= ~ones; }
        }
        if (lane_id() == 0) sc->tmax[wave_id()] = kth;
        __syncthreads();
        if (tid == 0) {
            uint32_t t = sc->tmax[0];
            for (int w = 1; w < kSelWaves; ++w)
                t = (k <= kWave) ? max(t, sc->tmax[w]) : min(t, sc->tmax[w]);
            sc->sh[5] = t;
        }
    }
    LSH_TRACE(2, 9);
    __syncthreads();
    LSH_TRACE(2, 10);
    const uint32_t tau = sc->sh[5];
    for (int i0 = tid; i0 < n; i0 += kSelThreads * 4) {
        uint64_t kk[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = i0 + q * kSelThreads;
            kk[q] = (i < n) ? src.key(i) : 0ull;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i0 + q * kSelThreads < n && (uint32_t)(kk[q] >> 32) >= tau) {
                const uint32_t pos = atomicAdd(&sc->sh[3], 1u);
                if (pos < (uint32_t)kSelListCap) sc->list[pos] = kk[q];
            }
        }
    }
    LSH_TRACE(2, 11);
    __syncthreads();
    LSH_TRACE(2, 12);
    int m = (int)sc->sh[3];
    if (m > kSelListCap) {
        // too many keys tie with tau: exact radix select into the list (k <= 256 fits)
        __syncthreads();
        block_radix_select(src, k, sc->list, sc);
        m = k;
    }
    // sort the m listed keys descending by rank counting; the first min(m, k) are the answer
    for (int e = tid; e < m; e += kSelThreads) {
        const uint64_t mine = sc->list[e];
        int rank = 0;
#pragma unroll 4
        for (int j = 0; j < m; ++j) rank += (sc->list[j] > mine) ? 1 : 0;
        if (rank < k) out[rank] = mine;
    }
    LSH_TRACE(2, 13);
    __syncthreads();
    LSH_TRACE(2, 14);
    return min(n, k);
}

// grid = R workgroups (one per hidden row).
__global__ void __launch_bounds__(kSelThreads)
k_select(const float* __restrict__ logits, int64_t cpitch, const int32_t* __restrict__ cand,
         const int32_t* __restrict__ count, int V, int B, const float* __restrict__ beam_scores,
         uint64_t* part, int32_t* part_n, float* lse_out, uint64_t* merge_keys, int32_t* tickets,
         int32_t* __restrict__ out_beam, int32_t* __restrict__ out_word,
         float* __restrict__ out_score) {
    __shared__ SelScratch sc;
    __shared__ uint64_t sel[256];
    __shared__ uint64_t mk_lds[kSelMergeLds];
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    const int r = blockIdx.x;
    const int s = r / B;
    LSH_TRACE(2, 0);
    const float* row = logits + (size_t)r * cpitch;
    // the first batch of the row is requested together with the candidate count: every address
    // lies inside the row's cpitch floats, whatever the count turns out to be
    float x[kSelBatch];
#pragma unroll
    for (int q = 0; q < kSelBatch; ++q) {
        const int c = tid + q * kSelThreads;
        x[q] = (c < cpitch) ? row[c] : 0.f;
    }
    const int C = count ? count[s] : V;

    // ---- one sweep: online log-sum-exp (Eq. 1 denominator) and this thread's largest logit ----
    float m = -INFINITY, sum = 0.f;
    uint32_t lmax = 0;
    for (int c0 = tid; c0 < C; c0 += kSelThreads * kSelBatch) {
        if (c0 != tid) {
#pragma unroll
            for (int q = 0; q < kSelBatch; ++q) {
                const int c = c0 + q * kSelThreads;
                x[q] = (c < C) ? row[c] : 0.f;
            }
        }
        float bm = -INFINITY;
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q)
            if (c0 + q * kSelThreads < C) bm = fmaxf(bm, x[q]);
        if (bm > m) { sum *= expf(m - bm); m = bm; }
#pragma unroll
        for (int q = 0; q < kSelBatch; ++q)
            if (c0 + q * kSelThreads < C) sum += expf(x[q] - m);
        lmax = max(lmax, f32_sortable(bm + 0.0f));
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, kWave), s2 = __shfl_xor(sum, off, kWave);
        const float mm = fmaxf(m, m2);
        const float a = (m == -INFINITY) ? 0.f : sum * expf(m - mm);
        const float b = (m2 == -INFINITY) ? 0.f : s2 * expf(m2 - mm);
        m = mm; sum = a + b;
    }
    if (ln == 0) { sc.redm[wv] = m; sc.reds[wv] = sum; }
    __syncthreads();
    float M = -INFINITY;
    for (int w = 0; w < kSelWaves; ++w) M = fmaxf(M, sc.redm[w]);
    float Ssum = 0.f;
    for (int w = 0; w < kSelWaves; ++w)
        if (sc.redm[w] != -INFINITY) Ssum += sc.reds[w] * expf(sc.redm[w] - M);
    const float lse = M + logf(Ssum);
    LSH_TRACE(2, 1);

    // ---- the row's B best logits, best first (second sweep re-reads the row from cache) -------
    const int nsel = block_topk_sorted(KeySrc{row, nullptr, C}, B, lmax, part + (size_t)r * B, &sc);
    if (tid == 0) { part_n[r] = nsel; lse_out[r] = lse; }
    LSH_TRACE(2, 2);

    // ---- last workgroup of the sentence merges ------------------------------------------------
    __threadfence();
    __syncthreads();
    if (tid == 0) sc.sh[4] = (uint32_t)atomicAdd(&tickets[s], 1);
    __syncthreads();
    LSH_TRACE(2, 3);
    if ((int)sc.sh[4] != B - 1) return;
    LSH_TRACE_ANY(2, 4);
    __threadfence();
    LSH_TRACE_ANY(2, 5);

    // keys of all B*B partial slots, every load independent of the others:
    // score = beam_score + (logit - lse); ties -> lower beam, then lower candidate position
    // (= lower word id, the list is ascending).  Unused slots get distinct keys below any score.
    const int nslots = B * B;
    uint64_t* mk = (nslots <= kSelMergeLds) ? mk_lds : merge_keys + (size_t)s * nslots;
    uint32_t lmax2 = 0;
    for (int idx = tid; idx < nslots; idx += kSelThreads) {
        const int i = idx / B, e = idx - i * B;
        const int rr = s * B + i;
        const int n_i = part_n[rr];
        const float lse_i = lse_out[rr];
        const float bs = beam_scores[rr];
        const uint64_t k = part[(size_t)rr * B + e];
        uint64_t out = (uint64_t)(~(uint32_t)idx);
        if (e < n_i) {
            const float score = bs + (key_value(k) - lse_i);
            out = make_key(score, ((uint32_t)i << 24) | key_index(k));
        }
        mk[idx] = out;
        lmax2 = max(lmax2, (uint32_t)(out >> 32));
    }
    __syncthreads();  // mk is read back by other threads of this workgroup below
    LSH_TRACE_ANY(2, 6);
    const int nfin = block_topk_sorted(KeySrc{nullptr, mk, nslots}, B, lmax2, sel, &sc);
    LSH_TRACE_ANY(2, 7);

    for (int e = tid; e < B; e += kSelThreads) {
        const size_t o = (size_t)s * B + e;
        float score = -INFINITY;
        uint32_t idx = 0;
        if (e < nfin && (uint32_t)(sel[e] >> 32) != 0u) {
            score = key_value(sel[e]);
            idx = key_index(sel[e]);
        }
        if (score == -INFINITY || score != score) {
            out_beam[o] = -1; out_word[o] = -1; out_score[o] = -INFINITY;
        } else {
            const int c = (int)(idx & 0xFFFFFFu);
            out_beam[o] = (int)(idx >> 24);
            out_word[o] = cand ? cand[(size_t)s * V + c] : c;
            out_score[o] = score;
        }
    }
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
