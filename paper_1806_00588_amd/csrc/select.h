// Log-softmax over the candidate list (Eq. 1 restricted to V_LSH) and beam expansion, on the
// device.  The paper copies P[B,|V|] to the host and heap-sorts there; here one workgroup per
// hidden row reduces its logits to (log-sum-exp, its B best columns), and the last workgroup of
// a sentence to finish merges the B partial lists into the sentence's B best (beam, word) pairs.
//
// A row's B best raw logits are a superset of what that row can contribute to the sentence's
// top B (score = beam_score + logit - lse is increasing in logit inside a row), so selection on
// raw logits loses nothing.
//
// Selection is an exact radix select on 64-bit keys that are distinct by construction:
//   high 32 bits: order-preserving image of the fp32 value; low 32 bits: ~(tie-break index),
// so "larger key" means "larger value, then lower index" and the k-th key is unique.
#pragma once
#include "device_utils.h"

namespace lshbeam {

constexpr int kSelThreads = 256;

struct SelScratch {            // LDS
    uint32_t hist[256];
    uint32_t sh[8];
    float redm[kSelThreads / kWave];
    float reds[kSelThreads / kWave];
};

// Writes the k largest of the n distinct keys key(0..n-1) to out[] (any order); returns how many
// were written (min(n, k)).  All threads of the workgroup must call it.
template <typename KeyFn>
__device__ int block_select_largest(KeyFn key, int n, int k, uint64_t* out, SelScratch* sc) {
    const int tid = threadIdx.x;
    if (n <= k) {
        for (int i = tid; i < n; i += kSelThreads) out[i] = key(i);
        __syncthreads();
        return n;
    }
    uint64_t prefix = 0, mask = 0;
    uint32_t remaining = (uint32_t)k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        sc->hist[tid] = 0;  // kSelThreads == 256 bins
        __syncthreads();
        for (int i = tid; i < n; i += kSelThreads) {
            const uint64_t kk = key(i);
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
    for (int i = tid; i < n; i += kSelThreads) {
        const uint64_t kk = key(i);
        if ((kk & mask) >= prefix) {
            const uint32_t pos = atomicAdd(&sc->sh[3], 1u);
            if (pos < (uint32_t)k) out[pos] = kk;
        }
    }
    __syncthreads();
    return k;
}

__device__ __forceinline__ uint64_t make_key(float v, uint32_t index) {
    return ((uint64_t)f32_sortable(v + 0.0f) << 32) | (uint64_t)(~index);
}
__device__ __forceinline__ float key_value(uint64_t k) { return sortable_f32((uint32_t)(k >> 32)); }
__device__ __forceinline__ uint32_t key_index(uint64_t k) { return ~(uint32_t)k; }

// grid = R workgroups (one per hidden row).
__global__ void __launch_bounds__(kSelThreads)
k_select(const float* __restrict__ logits, int64_t cpitch, const int32_t* __restrict__ cand,
         const int32_t* __restrict__ count, int V, int B, const float* __restrict__ beam_scores,
         uint64_t* part, int32_t* part_n, float* lse_out, uint64_t* merge_keys, int32_t* __restrict__ tickets,
         int32_t* __restrict__ out_beam, int32_t* __restrict__ out_word,
         float* __restrict__ out_score) {
    __shared__ SelScratch sc;
    __shared__ uint64_t sel[256];
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    const int r = blockIdx.x;
    const int s = r / B;
    const int C = count ? count[s] : V;
    const float* row = logits + (size_t)r * cpitch;

    // ---- log-sum-exp of the row (Eq. 1 denominator), online per thread then merged ----------
    float m = -INFINITY, sum = 0.f;
    for (int c = tid; c < C; c += kSelThreads) {
        const float x = row[c];
        if (x > m) { sum = sum * expf(m - x) + 1.f; m = x; }
        else sum += expf(x - m);
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
    for (int w = 0; w < kSelThreads / kWave; ++w) M = fmaxf(M, sc.redm[w]);
    float Ssum = 0.f;
    for (int w = 0; w < kSelThreads / kWave; ++w)
        if (sc.redm[w] != -INFINITY) Ssum += sc.reds[w] * expf(sc.redm[w] - M);
    const float lse = M + logf(Ssum);
    __syncthreads();

    // ---- the row's B best logits ------------------------------------------------------------
    auto row_key = [&](int c) { return make_key(row[c], (uint32_t)c); };
    const int nsel = block_select_largest(row_key, C, B, part + (size_t)r * B, &sc);
    if (tid == 0) { part_n[r] = nsel; lse_out[r] = lse; }

    // ---- last workgroup of the sentence merges ----------------------------------------------
    __threadfence();
    __syncthreads();
    if (tid == 0) sc.sh[4] = (uint32_t)atomicAdd(&tickets[s], 1);
    __syncthreads();
    if ((int)sc.sh[4] != B - 1) return;
    __threadfence();

    // keys of all partial entries: score = beam_score + (logit - lse); ties -> lower beam, then
    // lower candidate position (= lower word id, the list is ascending)
    uint64_t* mk = merge_keys + (size_t)s * B * B;
    int n = 0;
    for (int i = 0; i < B; ++i) {
        const int rr = s * B + i;
        const int n_i = part_n[rr];
        const float lse_i = lse_out[rr];
        const float bs = beam_scores[rr];
        for (int e = tid; e < n_i; e += kSelThreads) {
            const uint64_t k = part[(size_t)rr * B + e];
            const float score = bs + (key_value(k) - lse_i);
            mk[n + e] = make_key(score, ((uint32_t)i << 24) | key_index(k));
        }
        n += n_i;
    }
    __syncthreads();  // mk is read back by other threads of this workgroup below
    auto mkey = [&](int i) { return mk[i]; };
    const int nfin = block_select_largest(mkey, n, B, sel, &sc);

    // rank sort of the (at most B <= 256) winners, best first
    for (int e = tid; e < B; e += kSelThreads) {
        if (e < nfin) {
            const uint64_t k = sel[e];
            int rank = 0;
            for (int f = 0; f < nfin; ++f) rank += (sel[f] > k) ? 1 : 0;
            const float score = key_value(k);
            const uint32_t idx = key_index(k);
            const int beam = (int)(idx >> 24), c = (int)(idx & 0xFFFFFFu);
            const size_t o = (size_t)s * B + rank;
            if (score == -INFINITY || score != score) {
                out_beam[o] = -1; out_word[o] = -1; out_score[o] = -INFINITY;
            } else {
                out_beam[o] = beam;
                out_word[o] = cand ? cand[(size_t)s * V + c] : c;
                out_score[o] = score;
            }
        } else {
            const size_t o = (size_t)s * B + e;
            out_beam[o] = -1; out_word[o] = -1; out_score[o] = -INFINITY;
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
