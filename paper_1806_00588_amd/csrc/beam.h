// Beam bookkeeping around the decode step (Introduction, "Beam expansion"; Table 1, row "Hidden
// states reorder"): after the step has chosen, for every slot b of a sentence, a parent beam and
// a word, the recurrent state rows are gathered by parent, the choice is recorded for the final
// backtrace, and the score vector of the next step is prepared (a hypothesis that produced the
// end-of-sentence word, and an empty slot, get -inf: they are never expanded again).
#pragma once
#include "device_utils.h"

namespace lshbeam {

constexpr int kMaxBeamStates = 16;

struct BeamStatePtrs {  // passed by value: no device-side pointer table to allocate
    const float* in[kMaxBeamStates];
    float* out[kMaxBeamStates];
};

// grid = (S*B, max(n_states, 1)), 256 threads.  Workgroup (r, k) copies row parent(r) of state
// array k to row r of its output array; workgroups with k == 0 also write the history and the
// next score of slot r.
__global__ void __launch_bounds__(256)
k_beam_advance(BeamStatePtrs sp, int n_states, int state_dim, int B, int eos,
               const int32_t* __restrict__ out_beam, const int32_t* __restrict__ out_word,
               const float* __restrict__ out_score, int32_t* __restrict__ backptr_t,
               int32_t* __restrict__ words_t, float* __restrict__ scores_t,
               float* __restrict__ next_scores) {
    const int r = blockIdx.x, k = blockIdx.y;
    const int s = r / B;
    int parent = out_beam[r];
    if (parent >= B) parent = -1;  // not a slot of this sentence: treated as empty
    if (k == 0 && threadIdx.x == 0) {
        const int32_t w = out_word[r];
        const float sc = out_score[r];
        backptr_t[r] = parent;
        words_t[r] = w;
        scores_t[r] = sc;
        next_scores[r] = (parent < 0 || w == eos) ? -INFINITY : sc;
    }
    if (k >= n_states) return;
    float* dst = sp.out[k] + (size_t)r * state_dim;
    if (parent < 0) {  // empty slot: a defined value
        for (int i = threadIdx.x; i < state_dim; i += blockDim.x) dst[i] = 0.f;
        return;
    }
    const float* src = sp.in[k] + ((size_t)s * B + parent) * state_dim;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) == 0 && (state_dim & 3) == 0) {
        const float4* s4 = reinterpret_cast<const float4*>(src);
        float4* d4 = reinterpret_cast<float4*>(dst);
        for (int i = threadIdx.x; i < (state_dim >> 2); i += blockDim.x) d4[i] = s4[i];
    } else {
        for (int i = threadIdx.x; i < state_dim; i += blockDim.x) dst[i] = src[i];
    }
}

// grid = S, one wave per sentence.  Best finished hypothesis (a slot whose word is eos) over all
// recorded steps -- highest score, then earliest step, then lowest slot --, or, if none finished,
// the best slot of the last step; then its words by walking the parent pointers back to step 0.
__global__ void __launch_bounds__(kWave)
k_beam_backtrace(int S, int B, int eos, int n_steps, const int32_t* __restrict__ backptr,
                 const int32_t* __restrict__ words, const float* __restrict__ scores,
                 int max_len, int32_t* __restrict__ tokens /*[S, max_len]*/,
                 int32_t* __restrict__ length /*[S]*/, float* __restrict__ best_score /*[S]*/) {
    const int s = blockIdx.x, ln = lane_id();
    const size_t SB = (size_t)S * B;
    if (n_steps <= 0) {  // nothing recorded (the scans below assume at least one step)
        if (ln == 0) { length[s] = 0; best_score[s] = -INFINITY; }
        return;
    }
    // key: score first, then earlier step, then lower slot (larger key wins)
    auto better = [](float sa, int ia, float sb, int ib) { return sa > sb || (sa == sb && ia < ib); };
    float bsc = -INFINITY;
    int bidx = INT32_MAX;  // step * B + slot
    for (int pass = 0; pass < 2 && bidx == INT32_MAX; ++pass) {
        // pass 0: finished hypotheses of all steps; pass 1 (none finished): slots of the last step
        const int lo = pass ? (n_steps - 1) * B : 0, hi = n_steps * B;
        float lsc = -INFINITY;
        int lidx = INT32_MAX;
        for (int i = lo + ln; i < hi; i += kWave) {
            const int t = i / B, b = i - t * B;
            const size_t at = (size_t)t * SB + (size_t)s * B + b;
            const bool ok = backptr[at] >= 0 && backptr[at] < B && (pass == 1 || words[at] == eos);
            const float sc = scores[at];
            if (ok && sc == sc && sc > -INFINITY && better(sc, i, lsc, lidx)) { lsc = sc; lidx = i; }
        }
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const float osc = __shfl_xor(lsc, off, kWave);
            const int oidx = __shfl_xor(lidx, off, kWave);
            if (better(osc, oidx, lsc, lidx)) { lsc = osc; lidx = oidx; }
        }
        bsc = lsc;
        bidx = lidx;
    }
    if (ln != 0) return;
    if (bidx == INT32_MAX) {  // every slot empty
        length[s] = 0;
        best_score[s] = -INFINITY;
        return;
    }
    const int t_end = bidx / B;
    int cur = bidx - t_end * B;
    length[s] = t_end + 1;
    best_score[s] = bsc;
    for (int t = t_end; t >= 0; --t) {
        const size_t at = (size_t)t * SB + (size_t)s * B + cur;
        tokens[(size_t)s * max_len + t] = words[at];
        cur = backptr[at];
        if (cur < 0 || cur >= B) break;  // malformed history: stop rather than index out of bounds
    }
}

}  // namespace lshbeam
