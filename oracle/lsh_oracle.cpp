// CPU oracle for the LSH reduced-vocabulary softmax + beam expansion of Shi, Xu & Knight,
// "Fast Locality Sensitive Hashing for Beam Search on GPU".
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, single-threaded, deliberately
// slow implementation of what the decode step computes, written from the paper's definitions
// with the plainest containers available (std::unordered_map buckets, std::set unions, a binary
// heap for the top-B).  It shares no code, header, table or constant with the HIP library, and
// only tests, the smoke check and the benchmark's CPU-baseline leg may call it.
//
// Every function cites the passage it follows.  Floating point is fp64 throughout, except that
// the winner-take-all comparisons are taken on the stored fp32 / bf16 values themselves (the
// comparison of two stored values is exact in any wider type, so no precision is chosen there).
//
// Readings taken where the paper is silent (each is pinned by a CPU test):
//   * Permute_p(x)[k] = x[perm_p[k]] ("gather"), I_p = index of the largest of the first K
//     permuted entries (Eq. 4-5); ties go to the lowest k.
//   * Codes are stored 0-based; inside a band the first code sits in the most significant
//     bits (Table 5: codes (1,2) -> (00)(01) -> (0001)_2).  bits per code = ceil(log2 K).
//   * The softmax of Eq. 1 is normalised over the candidate list only; no bias, no temperature.
//   * Beam expansion takes, per sentence, the B best (beam, word) pairs by
//     beam_score + log-probability; equal scores order by lower beam, then lower word id.
//   * The candidate list is emitted in ascending word id.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <queue>
#include <set>
#include <unordered_map>
#include <vector>

namespace {

inline double load_elem(const void* base, int64_t idx, int dtype) {
    if (dtype == 0) return (double)((const float*)base)[idx];
    // bf16: the 16 stored bits are the top half of an fp32 pattern
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    std::memcpy(&f, &bits, 4);
    return (double)f;
}

inline int code_bits(int K) {
    int b = 0;
    while ((1 << b) < K) ++b;
    return b;
}

// Eq. 4-5: one winner-take-all code.  Sequential scan, strict '>' so the first maximum wins.
inline int wta_one(const void* x, int64_t row_off, int dtype, const int32_t* perm, int K) {
    int best = 0;
    double bestv = load_elem(x, row_off + perm[0], dtype);
    for (int k = 1; k < K; ++k) {
        double v = load_elem(x, row_off + perm[k], dtype);
        if (v > bestv) { bestv = v; best = k; }
    }
    return best;
}

// Eq. 6-8: band w concatenates codes w*u .. w*u+u-1, first code most significant.
inline int32_t band_of(const int32_t* codes, int w, int u, int bits) {
    int32_t b = 0;
    for (int i = 0; i < u; ++i) b = (b << bits) | codes[w * u + i];
    return b;
}

struct Index {
    const void* E;
    int V, d, dtype, P, K, W, u, bits;
    int64_t ld;
    std::vector<int32_t> perms;                                   // [P,K]
    std::vector<std::unordered_map<int32_t, std::vector<int32_t>>> T;  // T_w = {band code: [word ids]}
};

void band_codes_of_row(const Index* ix, const void* X, int64_t row_off, int dtype, int32_t* out) {
    std::vector<int32_t> codes(ix->P);
    for (int p = 0; p < ix->P; ++p)
        codes[p] = wta_one(X, row_off, dtype, &ix->perms[(size_t)p * ix->K], ix->K);
    for (int w = 0; w < ix->W; ++w) out[w] = band_of(codes.data(), w, ix->u, ix->bits);
}

struct Entry { double score; int32_t beam, word; };
// "a ranks before b": higher score, then lower beam id, then lower word id.
inline bool ranks_before(const Entry& a, const Entry& b) {
    if (a.score != b.score) return a.score > b.score;
    if (a.beam != b.beam) return a.beam < b.beam;
    return a.word < b.word;
}
struct WorstOnTop {  // priority_queue keeps the entry that ranks last at top()
    bool operator()(const Entry& a, const Entry& b) const { return ranks_before(a, b); }
};

}  // namespace

extern "C" {

// Eq. 4-5 for n vectors.  X is [n, ld] (dtype 0 = fp32, 1 = bf16 bit patterns), perms [P,K],
// codes_out [n,P], 0-based.
int orc_wta_codes(const void* X, int64_t n, int d, int64_t ld, int dtype, const int32_t* perms,
                  int P, int K, int32_t* codes_out) {
    if (!X || !perms || !codes_out || K < 1 || K > d) return 1;
    for (int64_t r = 0; r < n; ++r)
        for (int p = 0; p < P; ++p)
            codes_out[r * P + p] = wta_one(X, r * ld, dtype, perms + (size_t)p * K, K);
    return 0;
}

// Eq. 6-8.  codes [n,P] -> band_out [n,W]; requires P % W == 0 and u*bits <= 30 (the paper's
// "fits an int32" condition after Eq. 8).
int orc_band_codes(const int32_t* codes, int64_t n, int P, int W, int K, int32_t* band_out) {
    if (W < 1 || P % W) return 1;
    int u = P / W, bits = code_bits(K);
    if (u * bits > 30) return 1;
    for (int64_t r = 0; r < n; ++r)
        for (int w = 0; w < W; ++w) band_out[r * W + w] = band_of(codes + r * P, w, u, bits);
    return 0;
}

// Section "Cuckoo lookup", first step: hash every embedding row and file its id under its band
// code, one table per band.  (The paper then flattens T_w and indexes it with a cuckoo table;
// the mapping code -> word list is the same, and that mapping is all the oracle keeps.)
void* orc_build(const void* E, int V, int d, int64_t ld, int dtype, const int32_t* perms, int P,
                int K, int W) {
    if (!E || !perms || V < 1 || K < 1 || K > d || W < 1 || P % W) return nullptr;
    Index* ix = new Index();
    ix->E = E; ix->V = V; ix->d = d; ix->ld = ld; ix->dtype = dtype;
    ix->P = P; ix->K = K; ix->W = W; ix->u = P / W; ix->bits = code_bits(K);
    if (ix->u * ix->bits > 30) { delete ix; return nullptr; }
    ix->perms.assign(perms, perms + (size_t)P * K);
    ix->T.resize(W);
    std::vector<int32_t> bc(W);
    for (int j = 0; j < V; ++j) {
        band_codes_of_row(ix, E, (int64_t)j * ld, dtype, bc.data());
        for (int w = 0; w < W; ++w) ix->T[w][bc[w]].push_back(j);
    }
    return ix;
}

void orc_free(void* h) { delete (Index*)h; }

int orc_num_buckets(const void* h, int band) {
    const Index* ix = (const Index*)h;
    return (int)ix->T[band].size();
}

// All band codes present in table `band` (unordered).  Returns the number written.
int orc_bucket_keys(const void* h, int band, int32_t* keys_out, int cap) {
    const Index* ix = (const Index*)h;
    int n = 0;
    for (const auto& kv : ix->T[band]) { if (n < cap) keys_out[n] = kv.first; ++n; }
    return n;
}

// T_w[code]: returns the length (-1 if the code has no bucket) and writes up to cap ids.
int orc_bucket(const void* h, int band, int32_t code, int32_t* out, int cap) {
    const Index* ix = (const Index*)h;
    auto it = ix->T[band].find(code);
    if (it == ix->T[band].end()) return -1;
    int n = (int)it->second.size();
    for (int i = 0; i < n && i < cap; ++i) out[i] = it->second[i];
    return n;
}

// Band codes of hidden rows with the index's own permutations (H is fp32 [B,d], pitch d).
int orc_hidden_band_codes(const void* h, const float* H, int B, int32_t* out /*[B,W]*/) {
    const Index* ix = (const Index*)h;
    for (int i = 0; i < B; ++i)
        band_codes_of_row(ix, H, (int64_t)i * ix->d, 0, out + (size_t)i * ix->W);
    return 0;
}

// Algorithm 1 run for every (beam i, band w): L[i, word] += 1 for each word in the span that the
// band code of H_i selects.  This is Eq. 9 evaluated through the tables.  L is [B,V], zeroed here.
int orc_hit_counts(const void* h, const float* H, int B, int32_t* L) {
    const Index* ix = (const Index*)h;
    std::memset(L, 0, sizeof(int32_t) * (size_t)B * ix->V);
    std::vector<int32_t> bc(ix->W);
    for (int i = 0; i < B; ++i) {
        band_codes_of_row(ix, H, (int64_t)i * ix->d, 0, bc.data());
        for (int w = 0; w < ix->W; ++w) {
            auto it = ix->T[w].find(bc[w]);
            if (it == ix->T[w].end()) continue;
            for (int32_t word : it->second) L[(size_t)i * ix->V + word] += 1;
        }
    }
    return 0;
}

// Eq. 10 then Eq. 3:  V_LSH = V_T  U  { j : exists i with L[i,j] >= t }, as an ascending list.
// Returns |V_LSH| (writes at most cap ids).
int orc_candidates(const void* h, const float* H, int B, const int32_t* topfreq, int T, int t,
                   int32_t* out, int cap) {
    const Index* ix = (const Index*)h;
    std::vector<int32_t> L((size_t)B * ix->V);
    orc_hit_counts(h, H, B, L.data());
    std::set<int32_t> cand;
    for (int k = 0; k < T; ++k) cand.insert(topfreq[k]);
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < ix->V; ++j)
            if (L[(size_t)i * ix->V + j] >= t) cand.insert(j);
    int n = 0;
    for (int32_t j : cand) { if (n < cap) out[n] = j; ++n; }
    return n;
}

// Eq. 2 restricted to the candidate columns, then Eq. 1 as a log-probability normalised over
// those columns:  logit[i,c] = sum_k H[i,k] * E[cand[c],k]  (k ascending, fp64),
// lp[i,c] = logit[i,c] - (m_i + log sum_c' exp(logit[i,c'] - m_i)).
// cand == NULL means the identity list 0..C-1 (full vocabulary when C == V).
int orc_logprobs(const void* h, const float* H, int B, const int32_t* cand, int C,
                 double* logits /*[B,C] or NULL*/, double* lp /*[B,C]*/) {
    const Index* ix = (const Index*)h;
    for (int i = 0; i < B; ++i) {
        double* row = lp + (size_t)i * C;
        for (int c = 0; c < C; ++c) {
            int64_t j = cand ? cand[c] : c;
            double acc = 0.0;
            for (int k = 0; k < ix->d; ++k)
                acc += (double)H[(size_t)i * ix->d + k] * load_elem(ix->E, j * ix->ld + k, ix->dtype);
            row[c] = acc;
            if (logits) logits[(size_t)i * C + c] = acc;
        }
        if (C == 0) continue;
        double m = row[0];
        for (int c = 1; c < C; ++c) if (row[c] > m) m = row[c];
        double s = 0.0;
        for (int c = 0; c < C; ++c) s += std::exp(row[c] - m);
        double lse = m + std::log(s);
        for (int c = 0; c < C; ++c) row[c] -= lse;
    }
    return 0;
}

// Beam expansion (Introduction: heap selection over P in R^{B x |V|}, here over the candidate
// columns): the nsel best (beam, word) pairs by beam_scores[beam] + lp[beam, c], best first.
// Pairs whose score is -inf are never selected; missing entries are (-1, -1, -inf).
int orc_topb(const double* beam_scores, const double* lp, int B, const int32_t* cand, int C,
             int nsel, int32_t* out_beam, int32_t* out_word, double* out_score) {
    std::priority_queue<Entry, std::vector<Entry>, WorstOnTop> heap;
    const double ninf = -std::numeric_limits<double>::infinity();
    for (int i = 0; i < B; ++i) {
        for (int c = 0; c < C; ++c) {
            Entry e{beam_scores[i] + lp[(size_t)i * C + c], i, cand ? cand[c] : c};
            if (!(e.score > ninf)) continue;
            if ((int)heap.size() < nsel) heap.push(e);
            else if (ranks_before(e, heap.top())) { heap.pop(); heap.push(e); }
        }
    }
    int n = (int)heap.size();
    for (int r = n; r < nsel; ++r) { out_beam[r] = -1; out_word[r] = -1; out_score[r] = ninf; }
    for (int r = n - 1; r >= 0; --r) {
        out_beam[r] = heap.top().beam; out_word[r] = heap.top().word; out_score[r] = heap.top().score;
        heap.pop();
    }
    return n;
}

// One whole decode step for S sentences of B beams: candidates (or all of V when full_vocab),
// log-softmax, top-B.  H is fp32 [S*B, d]; beam_scores fp32 [S*B]; outputs [S,B]; counts [S].
int orc_decode_step(const void* h, const float* H, const float* beam_scores, const int32_t* topfreq,
                    int T, int t, int full_vocab, int S, int B, int32_t* out_beam,
                    int32_t* out_word, double* out_score, int32_t* counts) {
    const Index* ix = (const Index*)h;
    std::vector<int32_t> cand(ix->V);
    std::vector<double> lp, bs(B);
    for (int s = 0; s < S; ++s) {
        const float* Hs = H + (size_t)s * B * ix->d;
        int C;
        if (full_vocab) { C = ix->V; for (int j = 0; j < C; ++j) cand[j] = j; }
        else C = orc_candidates(h, Hs, B, topfreq, T, t, cand.data(), ix->V);
        lp.resize((size_t)B * C);
        orc_logprobs(h, Hs, B, cand.data(), C, nullptr, lp.data());
        for (int i = 0; i < B; ++i) bs[i] = (double)beam_scores[(size_t)s * B + i];
        orc_topb(bs.data(), lp.data(), B, cand.data(), C, B, out_beam + (size_t)s * B,
                 out_word + (size_t)s * B, out_score + (size_t)s * B);
        if (counts) counts[s] = C;
    }
    return 0;
}

}  // extern "C"
