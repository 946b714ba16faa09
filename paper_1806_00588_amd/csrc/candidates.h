// Winner-take-all hashing, cuckoo probe, bucket walk and candidate-list compaction.
//
//   k_band_codes  : band codes (Eq. 4-8) of n rows; used on E at build time and for inspection.
//   k_candidates  : one workgroup per sentence.  Hashes the sentence's B hidden rows, probes the
//                   per-band cuckoo tables (Algorithm 1, lines 1-2), walks the hit spans
//                   (lines 3-6) marking a V-bit presence bitmap held in LDS, ORs in the
//                   top-frequent words (Eq. 3) and compacts the bitmap into an ascending id list
//                   (Eq. 10 with t = 1).
//
// The paper keeps an integer hit matrix L[B,V] in global memory and compacts it with a shared-
// memory scan by lane 0 of each warp.  With t = 1 only "hit at least once" matters, so L
// collapses to one bit per word per sentence; V bits fit in LDS (25 KB at V = 200k), the marks
// are idempotent LDS atomic ORs, and compaction is a popcount + wave prefix sum.  Unequal span
// lengths (the paper's warp-divergence problem) are handled by flattening: span lengths are
// prefix-summed across all (row, band) pairs and the flat element range is dealt to threads
// evenly, each finding its span by binary search.
#pragma once
#include "device_utils.h"

namespace lshbeam {

// One slot of a cuckoo table: 16 bytes so a probe is a single 128-bit load.
struct __attribute__((aligned(16))) Slot {
    int32_t key;     // band code, or -1 when empty (codes are >= 0)
    uint32_t start;  // first position of the span in the band's flat word array
    uint32_t len;    // span length
    uint32_t pad;
};

// Per-band description of its cuckoo table: two multiplicative hashes over one slot array.
struct __attribute__((aligned(32))) BandMeta {
    uint32_t slot_off;  // first slot of this band in the concatenated slot array
    uint32_t shift;     // 32 - log2(capacity)
    uint32_t a0, b0, a1, b1;
    uint32_t pad0, pad1;
};

__host__ __device__ __forceinline__ uint32_t cuckoo_hash(uint32_t a, uint32_t b, uint32_t key,
                                                         uint32_t shift) {
    return (a * key + b) >> shift;
}

// Both slots are loaded unconditionally: no dependent second probe, no divergence.
__device__ __forceinline__ void cuckoo_find(const Slot* __restrict__ slots, const BandMeta& m,
                                            int32_t code, uint32_t* start, uint32_t* len) {
    const uint32_t h0 = cuckoo_hash(m.a0, m.b0, (uint32_t)code, m.shift);
    const uint32_t h1 = cuckoo_hash(m.a1, m.b1, (uint32_t)code, m.shift);
    const int4 s0 = *reinterpret_cast<const int4*>(slots + m.slot_off + h0);
    const int4 s1 = *reinterpret_cast<const int4*>(slots + m.slot_off + h1);
    const bool hit0 = s0.x == code, hit1 = s1.x == code;
    *start = hit0 ? (uint32_t)s0.y : (uint32_t)s1.y;
    *len = hit0 ? (uint32_t)s0.z : (hit1 ? (uint32_t)s1.z : 0u);
}

// Eq. 4-8 for one (row, band): u windowed argmaxes (strict '>', so the lowest k wins a tie),
// packed with the first code in the most significant bits.
template <typename ET>
__device__ __forceinline__ int32_t band_code_of(const ET* __restrict__ row,
                                                const int32_t* __restrict__ perms, int w, int u,
                                                int K, int bits) {
    int32_t code = 0;
    for (int i = 0; i < u; ++i) {
        const int32_t* pm = perms + (size_t)(w * u + i) * K;
        int best = 0;
        float bv = elem_f32(row + pm[0]);
        for (int k = 1; k < K; ++k) {
            const float v = elem_f32(row + pm[k]);
            if (v > bv) { bv = v; best = k; }
        }
        code = (code << bits) | best;
    }
    return code;
}

template <typename ET>
__global__ void __launch_bounds__(256)
k_band_codes(const ET* __restrict__ X, int64_t ld, int64_t n, const int32_t* __restrict__ perms,
             int P, int K, int W, int bits, int32_t* __restrict__ out) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * W) return;
    const int64_t row = idx / W;
    const int w = (int)(idx - row * W);
    out[idx] = band_code_of<ET>(X + row * ld, perms, w, P / W, K, bits);
}

constexpr int kCandThreads = 1024;
constexpr int kCandWaves = kCandThreads / kWave;
constexpr int kCandStage = 12288;  // hidden values staged in LDS per chunk of rows (floats)

// Rows of a sentence are processed in chunks small enough that the chunk's hidden rows fit the
// LDS stage and its (row, band) pairs fit one workgroup-wide scan.
__host__ __device__ inline int candidates_rows_per_chunk(int B, int d, int W) {
    int rows = kCandStage / d;
    if (rows > kCandThreads / W) rows = kCandThreads / W;
    if (rows > B) rows = B;
    return rows < 1 ? 1 : rows;
}

// LDS words k_candidates needs.  The stage always holds at least one hidden row.
// Words reserved for the V-bit bitmap: rounded to 4 so that what follows is 16-byte aligned.
__host__ __device__ inline int bitmap_words_padded(int V) { return (((V + 31) >> 5) + 3) & ~3; }

__host__ __device__ inline size_t candidates_lds_words(int V, int d, int P, int K) {
    const size_t nwords = (size_t)bitmap_words_padded(V);
    const size_t stage = (size_t)d > (size_t)kCandStage ? (size_t)d : (size_t)kCandStage;
    return nwords + stage + (size_t)P * K + 3 * (size_t)kCandThreads + 64;
}

// Branch-free search in an ascending LDS array of kCandThreads entries whose first entry is 0:
// the last index whose value is <= e.  Always ten steps, so two searches interleave well.
__device__ __forceinline__ int last_not_above(const uint32_t* pref, uint32_t e) {
    int lo = 0;
#pragma unroll
    for (int step = kCandThreads / 2; step >= 1; step >>= 1)
        if (pref[lo + step] <= e) lo += step;
    return lo;
}

// Marks the ids of a list in an LDS bitmap.  Ids that fall into the same bitmap word are OR-ed
// inside the wave first and one lane issues the atomic: same-address LDS atomics serialise, and
// frequent-word ids tend to be consecutive.  `first` is this thread's already loaded list[tid]
// (or -1).  Called by all kCandThreads threads.
__device__ __forceinline__ void mark_id_list(uint32_t* bm, int V, const int32_t* __restrict__ list,
                                             int T, int32_t first) {
    const int tid = threadIdx.x, ln = lane_id();
    for (int i0 = 0; i0 < T; i0 += kCandThreads) {
        const int i = i0 + tid;
        const int32_t id = (i0 == 0) ? first : ((i < T) ? list[i] : -1);
        const bool ok = id >= 0 && id < V;
        const uint32_t word = ok ? (uint32_t)(id >> 5) : 0xFFFFFFFFu;
        const uint32_t bit = ok ? (1u << (id & 31)) : 0u;
        uint64_t todo = __ballot(ok);
        bool grouped = true;
        while (todo && grouped) {
            const int leader = __ffsll((unsigned long long)todo) - 1;
            const uint32_t w0 = wave_read_lane(word, leader);
            const bool mine = ok && word == w0;
            const uint64_t grp = __ballot(mine);
            const uint32_t ored = wave_or(mine ? bit : 0u);
            if (ln == leader) atomicOr(&bm[w0], ored);
            todo &= ~grp;
            grouped = __popcll(grp) > 1;  // scattered ids: stop grouping, plain atomics below
        }
        if (ok && ((todo >> ln) & 1ull)) atomicOr(&bm[word], bit);
    }
}

// Arguments of candidate generation (everything k_candidates takes except its outputs).
struct CandArgs {
    const float* H;          // [S*B, d] hidden rows
    int B, d;
    const int32_t* perms;    // [P, K]
    int P, K, W, bits;
    const Slot* slots;
    const BandMeta* bands;   // [W]
    const int32_t* words;    // [W, V]
    int V;
    const int32_t* topfreq;  // [T]
    int T;
};

// Builds sentence s's presence bitmap (V bits, at smem[0 .. ceil(V/32))) in LDS: hashing, cuckoo
// probes, bucket walk and the top-frequent words.  Called by all kCandThreads threads of a
// workgroup with candidates_lds_words() words of LDS; ends with a workgroup barrier.
__device__ __forceinline__ void build_presence_bitmap(const CandArgs& a, int s, uint32_t* smem) {
    const float* __restrict__ H = a.H;
    const int B = a.B, d = a.d, P = a.P, K = a.K, W = a.W, bits = a.bits, V = a.V, T = a.T;
    const int32_t* __restrict__ perms = a.perms;
    const Slot* __restrict__ slots = a.slots;
    const BandMeta* __restrict__ bands = a.bands;
    const int32_t* __restrict__ words = a.words;
    const int32_t* __restrict__ topfreq = a.topfreq;
    const int nwords = (V + 31) >> 5;
    const int stage_words = d > kCandStage ? d : kCandStage;
    uint32_t* bm = smem;                                   // presence bitmap, V bits
    const int bmw = bitmap_words_padded(V);
    float* stage = reinterpret_cast<float*>(bm + bmw);     // the chunk's hidden rows [rows][d]
    int32_t* lperms = reinterpret_cast<int32_t*>(bm + bmw + stage_words);  // perms [P][K]
    uint32_t* p_start = bm + bmw + stage_words + P * K;    // span start of each pair in the chunk
    uint32_t* p_band = p_start + kCandThreads;             // its band
    uint32_t* p_pref = p_band + kCandThreads;              // exclusive prefix of span lengths
    uint32_t* wsum = p_pref + kCandThreads;                // scan scratch (>= kCandWaves + 1)

    const int tid = threadIdx.x;
    const int u = P / W;
    const int rows_per_chunk = candidates_rows_per_chunk(B, d, W);
    LSH_TRACE(0, 0);

    // Everything whose address is known up front is requested before anything is waited for:
    // this thread's band descriptor (its (row-in-chunk, band) pair is fixed), its first
    // top-frequent id, and its share of the first chunk of hidden rows.
    const uint32_t my_w = (uint32_t)(tid % W);
    const BandMeta my_meta = bands[my_w];
    int32_t tf_first = (tid < T) ? topfreq[tid] : -1;
    const float* H0 = H + (size_t)s * B * d;
    const bool vec_ok = (((uintptr_t)H0 | ((uintptr_t)d * 4)) & 15) == 0;
    float4 r0 = {}, r1 = {}, r2 = {}, r3 = {};
    {
        const int n4 = (min(rows_per_chunk, B) * d) >> 2;
        if (vec_ok && n4 > 0) {
            const float4* H4 = reinterpret_cast<const float4*>(H0);
            r0 = H4[min(tid, n4 - 1)];
            r1 = H4[min(tid + kCandThreads, n4 - 1)];
            r2 = H4[min(tid + 2 * kCandThreads, n4 - 1)];
            r3 = H4[min(tid + 3 * kCandThreads, n4 - 1)];
        }
    }
    const int32_t perm_first = (tid < P * K) ? perms[tid] : 0;
    __builtin_amdgcn_sched_barrier(0);  // keep the loads above where they are: issued first
    for (int i = tid; i < nwords; i += kCandThreads) bm[i] = 0u;
    if (tid < P * K) lperms[tid] = perm_first;
    for (int i = tid + kCandThreads; i < P * K; i += kCandThreads) lperms[i] = perms[i];
    __syncthreads();
    LSH_TRACE(0, 1);

    // Eq. 3: the top-frequent words are members of every candidate list.
    mark_id_list(bm, V, topfreq, T, tf_first);
    LSH_TRACE(0, 11);

    for (int row0 = 0; row0 < B; row0 += rows_per_chunk) {
        const int rows = min(rows_per_chunk, B - row0);
        // The chunk's hidden rows are contiguous: copy them to LDS with coalesced loads (a row's
        // P*K permuted coordinates touch nearly every cache line of the row anyway), so that the
        // permuted gathers of Eq. 5 are LDS reads and no global load depends on another.
        const float* Hc = H0 + (size_t)row0 * d;
        const int nval = rows * d;
        if (vec_ok) {
            const float4* H4 = reinterpret_cast<const float4*>(Hc);
            float4* S4 = reinterpret_cast<float4*>(stage);
            const int n4 = nval >> 2;
            for (int e0 = tid; e0 < n4; e0 += 4 * kCandThreads) {  // 4 independent loads in flight
                if (row0 != 0 || e0 != tid) {  // the very first batch is already in registers
                    r0 = H4[min(e0, n4 - 1)];
                    r1 = H4[min(e0 + kCandThreads, n4 - 1)];
                    r2 = H4[min(e0 + 2 * kCandThreads, n4 - 1)];
                    r3 = H4[min(e0 + 3 * kCandThreads, n4 - 1)];
                }
                S4[e0] = r0;
                if (e0 + kCandThreads < n4) S4[e0 + kCandThreads] = r1;
                if (e0 + 2 * kCandThreads < n4) S4[e0 + 2 * kCandThreads] = r2;
                if (e0 + 3 * kCandThreads < n4) S4[e0 + 3 * kCandThreads] = r3;
            }
        } else {
            for (int e = tid; e < nval; e += kCandThreads) stage[e] = Hc[e];
        }
        LSH_TRACE(0, 12);
        __syncthreads();
        LSH_TRACE(0, 2);

        // Eq. 4-5: one thread per (row, permutation) takes the windowed argmax from the staged
        // row (strict '>' in window order, so the lowest k wins a tie); codes go to LDS.  When
        // the chunk has more codes than threads, each pair's thread computes its own u codes.
        const int npairs = rows * W;
        const bool par_codes = rows * P <= kCandThreads;
        uint32_t* codes = p_pref;  // free until the scan below
        auto wta = [&](const float* sv, const int32_t* pm) {
            int best = 0;
            float bv = -INFINITY;
            bool first = true;
            for (int k0 = 0; k0 < K; k0 += 8) {  // 8 window entries per round of LDS reads
                int idx[8];
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) idx[j] = pm[min(k0 + j, K - 1)];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = sv[idx[j]];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (k0 + j < K && (first || v[j] > bv)) { bv = v[j]; best = k0 + j; }
                    first = false;
                }
            }
            return best;
        };
        if (par_codes) {
            if (tid < rows * P) {
                const int i = tid / P, p = tid - i * P;
                codes[tid] = (uint32_t)wta(stage + (size_t)i * d, lperms + (size_t)p * K);
            }
            __syncthreads();
        }
        // Eq. 6-8 (first code most significant), then Algorithm 1 lines 1-2 for this pair
        uint32_t start = 0, len = 0, w = 0;
        if (tid < npairs) {
            const int i = tid / W;
            w = my_w;
            int32_t code = 0;
            for (int q = 0; q < u; ++q) {
                const int best = par_codes
                    ? (int)codes[i * P + (int)w * u + q]
                    : wta(stage + (size_t)i * d, lperms + ((size_t)w * u + q) * K);
                code = (code << bits) | best;
            }
            cuckoo_find(slots, my_meta, code, &start, &len);
        }
        __syncthreads();  // codes[] aliases p_pref
        LSH_TRACE(0, 3);
        uint32_t total;
        const uint32_t incl = block_incl_scan(len, wsum, &total);
        LSH_TRACE(0, 4);
        p_start[tid] = start;
        p_band[tid] = w;
        p_pref[tid] = incl - len;
        __syncthreads();
        // Algorithm 1 lines 3-6 as a flat walk over all spans of the chunk: element e belongs
        // to the last pair whose exclusive prefix is <= e.  Two span reads in flight per thread.
        for (uint32_t e0 = tid; e0 < total; e0 += 2 * kCandThreads) {
            const uint32_t ea = e0, eb = min(e0 + (uint32_t)kCandThreads, total - 1);
            const int la = last_not_above(p_pref, ea), lb = last_not_above(p_pref, eb);
            const int32_t ida = words[(size_t)p_band[la] * V + p_start[la] + (ea - p_pref[la])];
            const int32_t idb = words[(size_t)p_band[lb] * V + p_start[lb] + (eb - p_pref[lb])];
            atomicOr(&bm[ida >> 5], 1u << (ida & 31));
            atomicOr(&bm[idb >> 5], 1u << (idb & 31));  // a clamped duplicate sets a set bit again
        }
        __syncthreads();
        LSH_TRACE(0, 5);
    }

}

// Compaction of a V-bit LDS bitmap into the ascending id list out[0..count) (Eq. 10's selection
// made dense; the paper's Fig. 5 step).  Each wave owns a contiguous range of bitmap words (a
// multiple of 64 of them); popcount + wave prefix sum give every lane the output offset of its
// word's ids.  A sparse word is expanded by its own lane (neighbouring lanes write neighbouring
// addresses).  Dense words -- the top-frequent ids usually fill whole words -- would make each
// lane write a long private run, 128 bytes apart from its neighbour's; they are expanded two at
// a time by 32 lanes each, one lane per bit, so that their stores are contiguous.
// Called by all kCandThreads threads; wsum is LDS scratch of >= kCandWaves words.
__device__ __forceinline__ void compact_bitmap(const uint32_t* bm, int nwords, uint32_t* wsum,
                                               int32_t* __restrict__ out,
                                               int32_t* __restrict__ count_out) {
    const int tid = threadIdx.x, wv = wave_id(), ln = lane_id();
    int per_wave = (nwords + kCandWaves - 1) / kCandWaves;
    per_wave = (per_wave + kWave - 1) / kWave * kWave;
    const int wbeg = wv * per_wave;
    const int wend = min(nwords, wbeg + per_wave);
    uint32_t cnt = 0;
    for (int i = wbeg + ln; i < wend; i += kWave) cnt += __popc(bm[i]);
    cnt = wave_sum(cnt);
    if (ln == 0) wsum[wv] = cnt;
    __syncthreads();
    uint32_t running = 0, total = 0;
    for (int i = 0; i < kCandWaves; ++i) {
        const uint32_t x = wsum[i];
        if (i < wv) running += x;
        total += x;
    }
    const int half = ln >> 5, hbit = ln & 31;
    for (int i0 = wbeg; i0 < wend; i0 += kWave) {
        const int i = i0 + ln;
        const uint32_t bitsw = (i < wend) ? bm[i] : 0u;
        const uint32_t c = __popc(bitsw);
        const uint32_t incl = wave_incl_scan(c);
        const uint32_t off = running + incl - c;
        const bool dense = c >= 12;
        uint64_t dmask = __ballot(dense);
        if (!dense) {
            uint32_t b = bitsw, o = off;
            while (b) {
                out[o++] = (i << 5) + (__ffs(b) - 1);
                b &= b - 1;
            }
        }
        while (dmask) {  // wave-uniform
            const int la = __ffsll((unsigned long long)dmask) - 1;
            dmask &= dmask - 1;
            const int lb = dmask ? __ffsll((unsigned long long)dmask) - 1 : la;
            const bool have_b = dmask != 0;
            dmask &= dmask - 1;  // no-op on zero
            const uint32_t wa = wave_read_lane(bitsw, la), wb = wave_read_lane(bitsw, lb);
            const uint32_t oa = wave_read_lane(off, la), ob = wave_read_lane(off, lb);
            const uint32_t wbits = half ? wb : wa;
            const uint32_t woff = half ? ob : oa;
            const int wlane = half ? lb : la;
            const bool set = ((wbits >> hbit) & 1u) && (half == 0 || have_b);
            const uint64_t bal = __ballot(set);
            const uint32_t hm = half ? (uint32_t)(bal >> 32) : (uint32_t)bal;
            const uint32_t pos = __popc(hm & ((1u << hbit) - 1u));
            if (set) out[woff + pos] = ((i0 + wlane) << 5) + hbit;
        }
        running += wave_read_lane(incl, kWave - 1);
    }
    if (tid == 0) *count_out = (int32_t)total;
}

// One workgroup per sentence.  Requires W <= kCandThreads.
__global__ void __launch_bounds__(kCandThreads)
k_candidates(CandArgs a, int32_t* __restrict__ cand, int32_t* __restrict__ count) {
    extern __shared__ uint32_t smem[];
    const int s = blockIdx.x;
    const int nwords = (a.V + 31) >> 5;
    uint32_t* wsum = smem + candidates_lds_words(a.V, a.d, a.P, a.K) - 64;
    build_presence_bitmap(a, s, smem);
    compact_bitmap(smem, nwords, wsum, cand + (size_t)s * a.V, count + s);
    LSH_TRACE(0, 6);
}

// ---------------------------------------------------------------------------------------------
// Threshold t > 1 (Eq. 9-10 in full): the hit matrix L[i, j] counts in how many bands row i and
// word j collide, and a word is a candidate iff some row reaches t.  One workgroup per hidden
// row keeps that row of L in LDS as 16-bit counters (the paper keeps L in global memory), walks
// the row's W spans with one wave per span (Algorithm 1; spans are long here -- ~V / 2^(u bits)
// words -- so a wave per span is load-balanced enough and needs no search), and leaves the
// row's thresholded bits as a V-bit bitmap in global memory.  A second kernel ORs the sentence's
// row bitmaps with the top-frequent words (Eq. 3) and compacts.
// ---------------------------------------------------------------------------------------------

// LDS words of k_hit_rows: counters (2 per word), the hidden row, codes (2 per word), spans.
__host__ __device__ inline size_t hit_rows_lds_words(int V, int d, int P, int W) {
    return ((size_t)V + 1) / 2 + (size_t)((d + 3) & ~3) + ((size_t)P + 1) / 2 + 2 * (size_t)W + 8;
}

// grid = S*B workgroups (one per hidden row).  Requires W < 65536 (16-bit counters).
__global__ void __launch_bounds__(kCandThreads)
k_hit_rows(CandArgs a, int t, uint32_t* __restrict__ row_bitmaps /*[S*B, nwords]*/) {
    extern __shared__ uint32_t smem[];
    const int V = a.V, d = a.d, P = a.P, K = a.K, W = a.W, bits = a.bits;
    const int u = P / W;
    const int nwords = (V + 31) >> 5;
    uint32_t* cnt32 = smem;                                            // V 16-bit counters
    float* rowv = reinterpret_cast<float*>(cnt32 + (V + 1) / 2);       // the hidden row
    uint16_t* codes = reinterpret_cast<uint16_t*>(rowv + ((d + 3) & ~3));
    uint32_t* sp_start = reinterpret_cast<uint32_t*>(codes) + (P + 1) / 2;
    uint32_t* sp_len = sp_start + W;
    const int r = blockIdx.x;
    const int tid = threadIdx.x, wv = wave_id(), ln = lane_id();
    const float* hrow = a.H + (size_t)r * d;

    for (int i = tid; i < d; i += kCandThreads) rowv[i] = hrow[i];
    for (int i = tid; i < (V + 1) / 2; i += kCandThreads) cnt32[i] = 0u;
    __syncthreads();

    // Eq. 4-5: one windowed argmax per permutation (strict '>' in window order)
    for (int p = tid; p < P; p += kCandThreads) {
        const int32_t* pm = a.perms + (size_t)p * K;
        int best = 0;
        float bv = -INFINITY;
        bool first = true;
        for (int k0 = 0; k0 < K; k0 += 8) {  // 8 window entries per round of loads
            int idx[8];
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) idx[j] = pm[min(k0 + j, K - 1)];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = rowv[idx[j]];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (k0 + j < K && (first || v[j] > bv)) { bv = v[j]; best = k0 + j; }
                first = false;
            }
        }
        codes[p] = (uint16_t)best;
    }
    __syncthreads();
    // Eq. 6-8 and Algorithm 1 lines 1-2: one band per thread
    for (int w = tid; w < W; w += kCandThreads) {
        int32_t code = 0;
        for (int q = 0; q < u; ++q) code = (code << bits) | codes[w * u + q];
        uint32_t start, len;
        cuckoo_find(a.slots, a.bands[w], code, &start, &len);
        sp_start[w] = start;
        sp_len[w] = len;
    }
    __syncthreads();
    // Algorithm 1 lines 3-6: L[i, word] += 1, one wave per span, two spans in flight
    for (int w0 = wv; w0 < W; w0 += 2 * kCandWaves) {
        const int w1 = w0 + kCandWaves;
        const uint32_t s0 = sp_start[w0], l0 = sp_len[w0];
        const uint32_t s1 = (w1 < W) ? sp_start[w1] : 0u, l1 = (w1 < W) ? sp_len[w1] : 0u;
        const int32_t* span0 = a.words + (size_t)w0 * V + s0;
        const int32_t* span1 = a.words + (size_t)min(w1, W - 1) * V + s1;
        for (uint32_t i = ln; i < max(l0, l1); i += kWave) {
            const int32_t id0 = (i < l0) ? span0[i] : -1;
            const int32_t id1 = (i < l1) ? span1[i] : -1;
            if (id0 >= 0) atomicAdd(&cnt32[id0 >> 1], 1u << (16 * (id0 & 1)));
            if (id1 >= 0) atomicAdd(&cnt32[id1 >> 1], 1u << (16 * (id1 & 1)));
        }
    }
    __syncthreads();
    // Eq. 10 for this row: bit j = (L[i, j] >= t); lane l of a wave looks at counter base + l
    const uint16_t* cnt16 = reinterpret_cast<const uint16_t*>(cnt32);
    uint32_t* out = row_bitmaps + (size_t)r * nwords;
    const int nchunks = (V + kWave - 1) / kWave;  // 64 words of the vocabulary = 2 bitmap words
    for (int c = wv; c < nchunks; c += kCandWaves) {
        const int j = c * kWave + ln;
        const bool hit = j < V && (int)cnt16[j] >= t;
        const uint64_t bal = __ballot(hit);
        if (ln == 0) out[2 * c] = (uint32_t)bal;
        if (ln == 32 && 2 * c + 1 < nwords) out[2 * c + 1] = (uint32_t)(bal >> 32);
    }
}

// grid = S workgroups: OR of the sentence's B row bitmaps and the top-frequent words, compacted.
__global__ void __launch_bounds__(kCandThreads)
k_union_compact(const uint32_t* __restrict__ row_bitmaps, int B, int V,
                const int32_t* __restrict__ topfreq, int T, int32_t* __restrict__ cand,
                int32_t* __restrict__ count) {
    extern __shared__ uint32_t smem[];  // nwords + 64 words
    const int s = blockIdx.x, tid = threadIdx.x;
    const int nwords = (V + 31) >> 5;
    uint32_t* bm = smem;
    uint32_t* wsum = smem + nwords;
    const int32_t tf_first = (tid < T) ? topfreq[tid] : -1;
    const uint32_t* rb = row_bitmaps + (size_t)s * B * nwords;
    for (int i = tid; i < nwords; i += kCandThreads) {
        uint32_t x = 0;
        for (int b = 0; b < B; ++b) x |= rb[(size_t)b * nwords + i];
        bm[i] = x;
    }
    __syncthreads();
    mark_id_list(bm, V, topfreq, T, tf_first);
    __syncthreads();
    compact_bitmap(bm, nwords, wsum, cand + (size_t)s * V, count + s);
}

}  // namespace lshbeam
