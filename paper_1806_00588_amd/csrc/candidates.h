// Winner-take-all hashing, cuckoo probe, bucket walk and candidate-list compaction.
//
//   k_band_codes  : band codes (Eq. 4-8) of n rows; used on E at build time and for inspection.
//   k_candidates  : one workgroup per sentence.  Hashes the sentence's B hidden rows, probes the
//                   per-band cuckoo tables (Algorithm 1, lines 1-2), walks the hit spans
//                   (lines 3-6) marking a V-bit presence bitmap held in LDS, ORs in the
//                   top-frequent words (Eq. 3) and compacts the bitmap into an ascending id list
//                   (Eq. 10 with t = 1).
//   k_part_bitmaps: the same hashing for a range of a sentence's rows, the bitmap left in global
//                   memory (sentences with many beams are hashed by several workgroups).
//   k_hit_rows    : hit threshold t > 1 (Eq. 9-10 in full): one workgroup per hidden row counts
//                   the row's collisions per word in LDS and leaves the thresholded bitmap.
//   k_union_compact: OR of a sentence's part / row bitmaps + top-frequent words + compaction.
//
// The paper keeps an integer hit matrix L[B,V] in global memory and compacts it with a shared-
// memory scan by lane 0 of each warp.  With t = 1 only "hit at least once" matters, so L
// collapses to one bit per word per sentence; V bits fit in LDS (25 KB at V = 200k), the marks
// are idempotent LDS atomic ORs, and compaction is a popcount + wave prefix sum.  Unequal span
// lengths (the paper's warp-divergence problem) are handled by flattening: span lengths are
// prefix-summed across all (row, band) pairs and the flat element range is dealt to threads
// evenly, each finding its span by binary search.
#pragma once
#include <type_traits>
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

// Both slots are loaded unconditionally: no dependent second probe, no divergence.  In two
// halves for callers that have other work to do while the loads are in flight.
__device__ __forceinline__ void cuckoo_load(const Slot* __restrict__ slots, const BandMeta& m,
                                            int32_t code, int4* s0, int4* s1) {
    const uint32_t h0 = cuckoo_hash(m.a0, m.b0, (uint32_t)code, m.shift);
    const uint32_t h1 = cuckoo_hash(m.a1, m.b1, (uint32_t)code, m.shift);
    *s0 = *reinterpret_cast<const int4*>(slots + m.slot_off + h0);
    *s1 = *reinterpret_cast<const int4*>(slots + m.slot_off + h1);
}
__device__ __forceinline__ void cuckoo_resolve(const int4& s0, const int4& s1, int32_t code,
                                               uint32_t* start, uint32_t* len) {
    const bool hit0 = s0.x == code, hit1 = s1.x == code;
    *start = hit0 ? (uint32_t)s0.y : (uint32_t)s1.y;
    *len = hit0 ? (uint32_t)s0.z : (hit1 ? (uint32_t)s1.z : 0u);
}
// The hit-count kernel (threshold t > 1) cuts the vocabulary into kHitSlices ranges of
// hit_slice_words(V) ids and gives every (hidden row, slice) its own workgroup.  Spans are sorted
// by id, so the part of a span that falls into slice q is contiguous; where slices 1, 2, 3 begin
// inside every span is computed once at build time and stored beside the slot (x, y, z of a
// uint4; positions relative to the span's start).
constexpr int kHitSlices = 4;
__host__ __device__ inline int hit_slice_words(int V) {  // ids per slice: a multiple of 128
    return (((V + kHitSlices - 1) / kHitSlices) + 127) & ~127;
}

// The probe restricted to vocabulary slice q: (start, len) of the span's part inside it.  The
// cut positions of both candidate slots are loaded along with the slots (no dependent load).
__device__ __forceinline__ void cuckoo_find_slice(const Slot* __restrict__ slots,
                                                  const uint4* __restrict__ cuts, const BandMeta& m,
                                                  int32_t code, int q, uint32_t* start, uint32_t* len) {
    const uint32_t h0 = cuckoo_hash(m.a0, m.b0, (uint32_t)code, m.shift);
    const uint32_t h1 = cuckoo_hash(m.a1, m.b1, (uint32_t)code, m.shift);
    const int4 s0 = *reinterpret_cast<const int4*>(slots + m.slot_off + h0);
    const int4 s1 = *reinterpret_cast<const int4*>(slots + m.slot_off + h1);
    const uint4 c0 = cuts[m.slot_off + h0], c1 = cuts[m.slot_off + h1];
    const bool hit0 = s0.x == code, hit1 = s1.x == code;
    const uint32_t st = hit0 ? (uint32_t)s0.y : (uint32_t)s1.y;
    const uint32_t ln = hit0 ? (uint32_t)s0.z : (hit1 ? (uint32_t)s1.z : 0u);
    const uint4 c = hit0 ? c0 : c1;
    const uint32_t lo = (q == 0) ? 0u : (q == 1) ? c.x : (q == 2) ? c.y : c.z;
    const uint32_t hi = (q == 0) ? c.x : (q == 1) ? c.y : (q == 2) ? c.z : ln;
    *start = st + min(lo, ln);
    *len = (ln && hi > lo) ? min(hi, ln) - min(lo, ln) : 0u;
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
// Hidden values staged in LDS per chunk of rows (floats): at least this much (or one row, if a row
// is longer), more when a step's sentences have more beams and LDS has room (the host decides per
// step and passes the size along: CandArgs::stage_words, a multiple of 4).
constexpr int kDirectFlag = 32;      // word of the scan scratch that holds the direct walk's verdict
constexpr int kCandStage = 12288;
constexpr int kCandStageRows = 32;   // a larger stage is sized for at most this many rows
__host__ __device__ inline int candidates_min_stage(int d) {
    return ((d > kCandStage ? d : kCandStage) + 3) & ~3;
}

// Rows of a sentence are processed in chunks small enough that the chunk's hidden rows fit the
// LDS stage and its (row, band) pairs fit one workgroup-wide scan.
__host__ __device__ inline int candidates_rows_per_chunk(int B, int d, int W, int stage_words) {
    int rows = stage_words / d;
    if (rows > kCandThreads / W) rows = kCandThreads / W;
    if (rows > B) rows = B;
    return rows < 1 ? 1 : rows;
}

// LDS words k_candidates needs.  The stage always holds at least one hidden row.
// Words reserved for the V-bit bitmap: rounded to 4 so that what follows is 16-byte aligned.
__host__ __device__ inline int bitmap_words_padded(int V) { return (((V + 31) >> 5) + 3) & ~3; }

__host__ __device__ inline size_t candidates_lds_words(int V, int P, int K, int stage_words) {
    return (size_t)bitmap_words_padded(V) + (size_t)stage_words + (size_t)P * K +
           3 * (size_t)kCandThreads + 64;
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
__device__ __forceinline__ void mark_ids_of_wave(uint32_t* bm, int V, int32_t id) {
    const int ln = lane_id();
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
// `second`: list[tid + kCandThreads] likewise (or -1; id_list_second() asks for it).
__device__ __forceinline__ int32_t id_list_second(const int32_t* __restrict__ list, int T) {
    const int i = (int)threadIdx.x + kCandThreads;
    return (T > kCandThreads && i < T) ? list[i] : -1;   // (a uniform branch for short lists)
}
template <bool SECOND = false>
__device__ __forceinline__ void mark_id_list(uint32_t* bm, int V, const int32_t* __restrict__ list,
                                             int T, int32_t first, int32_t second = -1) {
    // the first round (with SECOND, the first two) has its ids in registers: kept apart from the
    // loop so that it contains no load (and no wait that would also cover loads the caller has
    // in flight)
    if (T > 0) mark_ids_of_wave(bm, V, first);
    if (SECOND && T > kCandThreads) mark_ids_of_wave(bm, V, second);
    for (int i = (SECOND ? 2 : 1) * kCandThreads + (int)threadIdx.x; i - (int)threadIdx.x < T; i += kCandThreads)
        mark_ids_of_wave(bm, V, (i < T) ? list[i] : -1);
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
    const uint4* cuts;       // per slot: where the vocabulary slices 1, 2, 3 begin inside its span
    int stage_words;         // LDS words for the staged hidden rows (>= d, a multiple of 4)
    // derived on the host (set_derived), so that no division stands before the kernel's first loads
    int rows_chunk;          // candidates_rows_per_chunk(B, d, W, stage_words)
    int u;                   // P / W codes per band
};

inline void set_derived(CandArgs& a) {
    a.rows_chunk = candidates_rows_per_chunk(a.B, a.d, a.W, a.stage_words);
    a.u = a.P / a.W;
}

// Builds sentence s's presence bitmap (V bits, at smem[0 .. ceil(V/32))) in LDS: hashing, cuckoo
// probes, bucket walk and the top-frequent words.  Only the sentence's rows [row_begin, row_end)
// are hashed (row_end < 0: all B).  Called by all kCandThreads threads of a workgroup with
// candidates_lds_words() words of LDS; ends with a workgroup barrier.
// DEEP (for the kernels that have the registers): walks of more than eight elements per thread
// keep twelve span reads in flight, and the second thousand of top-frequent ids is asked for up
// front too.
template <bool DEEP = false>
__device__ __forceinline__ void build_presence_bitmap(const CandArgs& a, int s, uint32_t* smem,
                                                      int row_begin = 0, int row_end = -1) {
    const float* __restrict__ H = a.H;
    const int B = a.B, d = a.d, P = a.P, K = a.K, W = a.W, bits = a.bits, V = a.V, T = a.T;
    const int32_t* __restrict__ perms = a.perms;
    const Slot* __restrict__ slots = a.slots;
    const BandMeta* __restrict__ bands = a.bands;
    const int32_t* __restrict__ words = a.words;
    const int32_t* __restrict__ topfreq = a.topfreq;
    const int nwords = (V + 31) >> 5;
    const int stage_words = a.stage_words;
    uint32_t* bm = smem;                                   // presence bitmap, V bits
    const int bmw = bitmap_words_padded(V);
    float* stage = reinterpret_cast<float*>(bm + bmw);     // the chunk's hidden rows [rows][d]
    int32_t* lperms = reinterpret_cast<int32_t*>(bm + bmw + stage_words);  // perms [P][K]
    uint32_t* p_start = bm + bmw + stage_words + P * K;    // span start of each pair in the chunk
    uint32_t* p_band = p_start + kCandThreads;             // its band
    uint32_t* p_pref = p_band + kCandThreads;              // exclusive prefix of span lengths
    uint32_t* wsum = p_pref + kCandThreads;                // scan scratch (>= kCandWaves + 1)

    const int tid = threadIdx.x;
    const int u = a.u;
    const int rows_per_chunk = a.rows_chunk;
    if (row_end < 0) row_end = B;
    LSH_TRACE(0, 0);
    LSH_TRACE_WG(0);

    // Everything whose address is known up front is requested before anything is waited for:
    // this thread's band descriptor (its (row-in-chunk, band) pair is fixed), its first
    // top-frequent id, and its share of the first chunk of hidden rows.
    const uint32_t my_w = (uint32_t)(tid - small_div(tid, W) * W);   // (tid < 1024, W <= P <= 1024)
    const BandMeta my_meta = bands[my_w];
    const int32_t tf_first = (tid < T) ? topfreq[tid] : -1;
    const int32_t tf_second = DEEP ? id_list_second(topfreq, T) : -1;
    const float* H0 = H + (size_t)s * B * d;
    const bool vec_ok = (((uintptr_t)H0 | ((uintptr_t)d * 4)) & 15) == 0;
    float4 r0 = {}, r1 = {}, r2 = {}, r3 = {};
    {
        const int n4 = (min(rows_per_chunk, row_end - row_begin) * d) >> 2;
        if (vec_ok && n4 > 0) {
            const float4* H4 = reinterpret_cast<const float4*>(H0 + (size_t)row_begin * d);
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
    LSH_TRACE(0, 1);
    // (no barrier here: the first chunk's staging barrier below also covers the cleared bitmap
    // and the staged permutations)
    bool topfreq_marked = false;

    for (int row0 = row_begin; row0 < row_end; row0 += rows_per_chunk) {
        const int rows = min(rows_per_chunk, row_end - row0);
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
                if (row0 != row_begin || e0 != tid) {  // the very first batch is already in registers
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
        if (tid == 0) wsum[kDirectFlag] = 0u;   // "a span of this chunk is too long for the direct walk"
        __syncthreads();
        LSH_TRACE(0, 2);
        LSH_TRACE_WG(1);

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
                const int i = small_div(tid, P), p = tid - i * P;
                codes[tid] = (uint32_t)wta(stage + (size_t)i * d, lperms + (size_t)p * K);
            }
            __syncthreads();
        }
        // Eq. 6-8 (first code most significant), then Algorithm 1 lines 1-2 for this pair
        uint32_t start = 0, len = 0, w = 0;
        int32_t code = 0;
        int4 slot0, slot1;
        if (tid < npairs) {
            const int i = small_div(tid, W);
            w = my_w;
            for (int q = 0; q < u; ++q) {
                const int best = par_codes
                    ? (int)codes[i * P + (int)w * u + q]
                    : wta(stage + (size_t)i * d, lperms + ((size_t)w * u + q) * K);
                code = (code << bits) | best;
            }
        }
        // (threads without a pair probe code 0 of their band and drop the result: a load inside
        // the branch would have to be waited for where the branch ends)
        cuckoo_load(slots, my_meta, code, &slot0, &slot1);
        // Eq. 3: the top-frequent words are members of every candidate list.  Marked here, while
        // the first chunk's probes are on their way (the bitmap was cleared before the staging
        // barrier; every consumer of the bitmap comes after the barrier that ends the chunk).
        if (!topfreq_marked) {
            mark_id_list<DEEP>(bm, V, topfreq, T, tf_first, tf_second);
            topfreq_marked = true;
            LSH_TRACE(0, 11);
        }
        // (the compiler would otherwise compare the slots -- and wait for them -- right after
        // the loads, before the marking; this pins their first use here)
        asm volatile("" : "+v"(slot0.x), "+v"(slot0.y), "+v"(slot0.z), "+v"(slot1.x), "+v"(slot1.y),
                          "+v"(slot1.z) :: "memory");
        if (tid < npairs) cuckoo_resolve(slot0, slot1, code, &start, &len);
        // Short spans are walked without the scan and the search below: kCandThreads / npairs
        // threads share a span, each taking every subs-th aligned group of four ids of the flat
        // word array (the array is padded, so a group may reach past a span's end but never past
        // the allocation), at most kDirectGroups groups per thread.  One span too long for that:
        // the flat walk for the whole chunk.
        constexpr int kDirectGroups = 4;
        const int subs = kCandThreads / npairs;
        {
            const size_t flat = (size_t)w * V + start;
            const uint32_t mis = (uint32_t)flat & 3u;
            p_start[tid] = (uint32_t)(flat >> 2);               // first group (W * V < 2^34)
            p_band[tid] = len | (mis << 30);                    // (len <= V <= 2^24)
            if (((len + mis + 3) >> 2) > (uint32_t)(subs * kDirectGroups)) wsum[kDirectFlag] = 1u;
        }
        __syncthreads();  // codes[] aliases p_pref
        LSH_TRACE(0, 3);
        LSH_TRACE_WG(2);
        if (wsum[kDirectFlag] == 0u) {   // (uniform)
            const int sub = small_div(tid, npairs), pair = tid - sub * npairs;
            const uint32_t g0 = p_start[pair], lm = p_band[pair];
            const uint32_t slen = lm & 0x3FFFFFFFu, smis = lm >> 30;
            const uint32_t ngroups = (sub < subs && slen) ? (slen + smis + 3) >> 2 : 0u;
            const int4* __restrict__ words4 = reinterpret_cast<const int4*>(words);
            int4 grp[kDirectGroups];
#pragma unroll
            for (int j = 0; j < kDirectGroups; ++j) {
                const uint32_t g = (uint32_t)(sub + subs * j);
                if (j > 0 && __ballot(g < ngroups) == 0ull) { grp[j] = make_int4(0, 0, 0, 0); continue; }   // (uniform)
                grp[j] = words4[(size_t)g0 + (g < ngroups ? g : 0u)];
            }
#pragma unroll
            for (int j = 0; j < kDirectGroups; ++j) {
                const uint32_t g = (uint32_t)(sub + subs * j);
                if (__ballot(g < ngroups) == 0ull) continue;   // (uniform)
                const uint32_t p0 = 4u * g;                    // position of the group's first id in the span + smis
                const int32_t ids[4] = {grp[j].x, grp[j].y, grp[j].z, grp[j].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (g < ngroups && p0 + c >= smis && p0 + c < smis + slen)
                        atomicOr(&bm[ids[c] >> 5], 1u << (ids[c] & 31));
            }
            __syncthreads();
            LSH_TRACE(0, 5);
            LSH_TRACE_WG(3);
            continue;
        }
        uint32_t total;
        const uint32_t incl = block_incl_scan(len, wsum, &total);
        LSH_TRACE(0, 4);
        p_start[tid] = start;
        p_band[tid] = w;
        p_pref[tid] = incl - len;
        __syncthreads();
        // Algorithm 1 lines 3-6 as a flat walk over all spans of the chunk: element e belongs
        // to the last pair whose exclusive prefix is <= e.  An index past the end is clamped for
        // the load and skipped for the mark: hundreds of atomics on the last element's word
        // would serialise.  Long walks (several elements per thread) keep four span reads in
        // flight per thread (twelve beyond eight elements per thread: a round is a trip to
        // memory), short ones two: with four, every thread searches four times even when the
        // chunk has fewer elements than that.
        auto walk = [&](auto width_tag) {
            constexpr int NW = decltype(width_tag)::value;
            for (uint32_t e0 = tid; e0 < total; e0 += NW * kCandThreads) {
                uint32_t e[NW];
                int l[NW];
                int32_t id[NW];
#pragma unroll
                for (int q = 0; q < NW; ++q) e[q] = min(e0 + (uint32_t)(q * kCandThreads), total - 1);
#pragma unroll
                for (int q = 0; q < NW; ++q) l[q] = last_not_above(p_pref, e[q]);
#pragma unroll
                for (int q = 0; q < NW; ++q)
                    id[q] = words[(size_t)p_band[l[q]] * V + p_start[l[q]] + (e[q] - p_pref[l[q]])];
#pragma unroll
                for (int q = 0; q < NW; ++q)
                    if (e0 + (uint32_t)(q * kCandThreads) < total)
                        atomicOr(&bm[id[q] >> 5], 1u << (id[q] & 31));
            }
        };
        if (DEEP && total > 8u * kCandThreads) walk(std::integral_constant<int, 12>{});
        else if (total > 4u * kCandThreads) walk(std::integral_constant<int, 4>{});
        else walk(std::integral_constant<int, 2>{});
        __syncthreads();
        LSH_TRACE(0, 5);
        LSH_TRACE_WG(3);
    }
    if (!topfreq_marked) {  // no rows to hash
        __syncthreads();
        mark_id_list<DEEP>(bm, V, topfreq, T, tf_first, tf_second);
        __syncthreads();
    }
}

// Compaction of a V-bit LDS bitmap into the ascending id list out[0..count) (Eq. 10's selection
// made dense; the paper's Fig. 5 step).  Each wave owns a contiguous range of bitmap words (a
// multiple of 64 of them); popcount + wave prefix sum give every lane the output offset of its
// word's ids.  A sparse word is expanded by its own lane (neighbouring lanes write neighbouring
// addresses).  Dense words -- the top-frequent ids usually fill whole words, and they sit next
// to each other, in one wave's range -- would make each lane write a long private run, 128 bytes
// apart from its neighbour's, and that one wave would expand them all: they are put on a list
// in LDS instead (word, output offset) and, after a barrier, expanded by ALL waves, 32 lanes per
// word, one lane per bit, so that the stores are contiguous.  Dense words beyond the list's
// capacity are expanded by their own wave, two at a time.
// Called by all kCandThreads threads; wsum is LDS scratch of >= kCandWaves + 1 words, dlist LDS
// room for dcap entries.
__device__ __forceinline__ void compact_bitmap(const uint32_t* bm, int nwords, uint32_t* wsum,
                                               uint2* dlist, int dcap, int32_t* __restrict__ out,
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
    if (tid == 0) wsum[kCandWaves] = 0;  // entries on the dense list
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
        if (dmask) {  // wave-uniform
            uint32_t base = 0;
            if (ln == 0) base = atomicAdd(&wsum[kCandWaves], (uint32_t)__popcll(dmask));
            base = wave_read_lane(base, 0);
            const uint32_t pos = base + lanes_below(dmask);
            const bool listed = dense && pos < (uint32_t)dcap;
            if (listed) dlist[pos] = make_uint2((uint32_t)i, off);
            dmask = __ballot(dense && !listed);
        }
        while (dmask) {  // wave-uniform: what the list had no room for
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
            const uint32_t pos = __popc(wbits & ((1u << hbit) - 1u));
            if (set) out[woff + pos] = ((i0 + wlane) << 5) + hbit;
        }
        running += wave_read_lane(incl, kWave - 1);
    }
    if (tid == 0) *count_out = (int32_t)total;
    __syncthreads();
    // the listed dense words: half a wave per word, all waves
    const int nlisted = (int)min(wsum[kCandWaves], (uint32_t)dcap);
    for (int k = 2 * wv + half; k < nlisted; k += 2 * kCandWaves) {
        const uint2 ent = dlist[k];
        const uint32_t wbits = bm[ent.x];
        const uint32_t pos = __popc(wbits & ((1u << hbit) - 1u));
        if ((wbits >> hbit) & 1u) out[ent.y + pos] = (int32_t)((ent.x << 5) + (uint32_t)hbit);
    }
}

// LDS of k_union_compact: the bitmap (rounded to an even number of words), 64 words of scan
// scratch, the dense-word list of compact_bitmap.
constexpr int kUnionDenseCap = 2048;
__host__ __device__ inline size_t union_compact_lds_words(int V) {
    return (size_t)bitmap_words_padded(V) + 64 + 2 * (size_t)kUnionDenseCap;
}

// One workgroup per sentence.  Requires W <= kCandThreads.
__global__ void __launch_bounds__(kCandThreads)
k_candidates(CandArgs a, int32_t* __restrict__ cand, int32_t* __restrict__ count) {
    extern __shared__ uint32_t smem[];
    const int s = blockIdx.x;
    const int nwords = (a.V + 31) >> 5;
    uint32_t* wsum = smem + candidates_lds_words(a.V, a.P, a.K, a.stage_words) - 64;
    build_presence_bitmap<true>(a, s, smem);
    // (the staged hidden rows are no longer needed: their room takes the dense-word list)
    uint2* dlist = reinterpret_cast<uint2*>(smem + bitmap_words_padded(a.V));
    compact_bitmap(smem, nwords, wsum, dlist, a.stage_words / 2, cand + (size_t)s * a.V, count + s);
    LSH_TRACE(0, 6);
}

// Sentences with many beams: the hidden rows of a sentence are hashed a chunk at a time, so one
// workgroup per sentence serialises ceil(B / rows per chunk) rounds of dependent memory round
// trips.  Here the sentence is cut into `nparts` parts of `part_rows` rows, one workgroup each;
// every part leaves its own V-bit bitmap (without the top-frequent words) in global memory at
// part_bitmaps[(s * nparts + part) * ceil(V/32)], and the consumer ORs the parts (Eq. 3's union).
__global__ void __launch_bounds__(kCandThreads)
k_part_bitmaps(CandArgs a, int part_rows, int nparts, uint32_t* __restrict__ part_bitmaps) {
    extern __shared__ uint32_t smem[];
    const int s = blockIdx.x / nparts, part = blockIdx.x - s * nparts;
    const int nwords = (a.V + 31) >> 5;
    a.T = 0;
    build_presence_bitmap<true>(a, s, smem, part * part_rows, min(a.B, (part + 1) * part_rows));
    uint32_t* out = part_bitmaps + (size_t)blockIdx.x * nwords;
    for (int i = threadIdx.x; i < nwords; i += kCandThreads) out[i] = smem[i];
}

// ---------------------------------------------------------------------------------------------
// Threshold t > 1 (Eq. 9-10 in full): the hit matrix L[i, j] counts in how many bands row i and
// word j collide, and a word is a candidate iff some row reaches t.  One workgroup per (hidden
// row, vocabulary slice) keeps its part of that row of L in LDS as 16-bit counters (the paper
// keeps L in global memory), adds one for every id of the row's W hit spans that falls into the
// slice (Algorithm 1), and leaves the thresholded bits as its part of the row's V-bit bitmap in
// global memory.  The consumer ORs the sentence's row bitmaps with the top-frequent words
// (Eq. 3).
// ---------------------------------------------------------------------------------------------

// LDS words of k_hit_rows without its load list: counters (2 per word, in blocks of 64 ids), the
// hidden row, codes (2 per word), scan scratch, three per-span arrays.
__host__ __device__ inline size_t hit_rows_fixed_lds_words(int V, int d, int P) {
    return (size_t)hit_slice_words(V) / 2 + (size_t)((d + 3) & ~3) + ((size_t)P + 1) / 2 + 32 +
           3 * (size_t)kCandThreads + 64;
}
constexpr int kHitListMin = 2048, kHitListMax = 16384;  // load-list entries per pass

// grid = S*B*kHitSlices workgroups (hidden row r = block / kHitSlices, slice q = block %
// kHitSlices).  Requires W <= kCandThreads (one span per thread), W * V < 2^30 (a 16-byte group
// index and a 4-bit mask share a word) and list_cap >= kHitListMin.
__global__ void __launch_bounds__(kCandThreads)
k_hit_rows(CandArgs a, int t, int list_cap, uint32_t* __restrict__ row_bitmaps /*[S*B, nwords]*/) {
    extern __shared__ uint32_t smem[];
    const int V = a.V, d = a.d, P = a.P, K = a.K, W = a.W, bits = a.bits;
    const int u = P / W;
    const int nwords = (V + 31) >> 5;
    const int Vq = hit_slice_words(V);                                 // ids of a slice
    uint32_t* cnt32 = smem;                                            // Vq 16-bit counters
    const int ncnt = Vq / 2;                                           // counter words
    float* rowv = reinterpret_cast<float*>(cnt32 + ncnt);              // the hidden row
    uint16_t* codes = reinterpret_cast<uint16_t*>(rowv + ((d + 3) & ~3));
    uint32_t* wsum = reinterpret_cast<uint32_t*>(codes) + (P + 1) / 2;  // scan scratch
    uint32_t* sp_pref = wsum + 32;                 // first list entry of each span (+ the total)
    uint32_t* sp_where = sp_pref + kCandThreads + 64;  // first 16-byte group << 2 | misalignment
    uint32_t* sp_len = sp_where + kCandThreads;
    uint32_t* list = sp_len + kCandThreads;        // load list [list_cap]
    const int r = blockIdx.x / kHitSlices, slice = blockIdx.x % kHitSlices;
    const int id0 = slice * Vq;                                        // first id of the slice
    const int tid = threadIdx.x, wv = wave_id(), ln = lane_id();
    const float* hrow = a.H + (size_t)r * d;

    LSH_TRACE(3, 0);
    // this thread's band descriptor is needed only after the codes: request it now
    const BandMeta my_meta = a.bands[min(tid, W - 1)];
    for (int i = tid; i < d; i += kCandThreads) rowv[i] = hrow[i];
    for (int i = tid; i < ncnt; i += kCandThreads) cnt32[i] = 0u;
    __syncthreads();
    LSH_TRACE(3, 1);

    // Eq. 4-5: one windowed argmax per permutation (strict '>' in window order, so the lowest k
    // wins a tie); window entries are fetched eight at a time, as 16-byte loads when K allows
    const bool pvec = (K & 3) == 0 && ((uintptr_t)a.perms & 15) == 0;
    for (int p = tid; p < P; p += kCandThreads) {
        const int32_t* pm = a.perms + (size_t)p * K;
        int best = 0;
        float bv = -INFINITY;
        bool first = true;
        for (int k0 = 0; k0 < K; k0 += 8) {
            int idx[8];
            float v[8];
            if (pvec) {
                const int4 q0 = *reinterpret_cast<const int4*>(pm + k0);
                const int4 q1 = *reinterpret_cast<const int4*>(pm + min(k0 + 4, K - 4));
                idx[0] = q0.x; idx[1] = q0.y; idx[2] = q0.z; idx[3] = q0.w;
                idx[4] = q1.x; idx[5] = q1.y; idx[6] = q1.z; idx[7] = q1.w;
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) idx[j] = pm[min(k0 + j, K - 1)];
            }
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
    LSH_TRACE(3, 2);

    // Eq. 6-8 and Algorithm 1 lines 1-2: thread w packs band w's code and probes its table.
    // Span ids are read in aligned groups of four (one 16-byte load): the span covers
    // `ngroups` of them starting at group `grp0` of the flat word array, its first id sitting
    // at position `mis` of the first group.
    uint32_t grp0 = 0, mis = 0, len = 0, ngroups = 0;
    if (tid < W) {
        int32_t code = 0;
        for (int q = 0; q < u; ++q) code = (code << bits) | codes[tid * u + q];
        uint32_t start;
        cuckoo_find_slice(a.slots, a.cuts, my_meta, code, slice, &start, &len);
        if (len) {
            const size_t g0 = (size_t)tid * V + start;
            grp0 = (uint32_t)(g0 >> 2);
            mis = (uint32_t)(g0 & 3);
            ngroups = (mis + len + 3) >> 2;
        }
    }
    uint32_t total;
    const uint32_t first_entry = block_incl_scan(ngroups, wsum, &total) - ngroups;
    sp_pref[tid] = (tid < W) ? first_entry : total;
    if (tid == 0) sp_pref[kCandThreads] = total;
    sp_where[tid] = (grp0 << 2) | mis;
    sp_len[tid] = len;
    __syncthreads();
    LSH_TRACE(3, 3);

    // Algorithm 1 lines 3-6: L[i, word] += 1 for every id of every hit span.  Spans have unequal
    // lengths (the source of the paper's divergence problem): they are flattened into a list of
    // 16-byte loads in LDS -- entry = group index << 4 | which of its four ids belong to the
    // span.  Every thread writes an equal, contiguous share of the list (it finds the span of
    // its first entry by search and walks on from there), and the workgroup then consumes the
    // list interleaved, kHitInFlight loads per thread in flight.  Lists longer than list_cap
    // are handled in passes.
    const int4* words4 = reinterpret_cast<const int4*>(a.words);
    constexpr int kHitInFlight = 8;
    // Counter of word id: 64 consecutive ids share 32 LDS words, id & 31 picks the word and bit 5
    // of the id its half, so that the thresholding pass below gets whole bitmap words from a
    // ballot over the low halves and one over the high halves.
    auto bump = [&](int32_t id, uint32_t ok) {
        id -= id0;  // position inside the slice (masked-out ids of neighbouring spans may be outside)
        if (ok) atomicAdd(&cnt32[((id >> 6) << 5) | (id & 31)], (id & 32) ? 0x10000u : 1u);
    };
    for (uint32_t pass0 = 0; pass0 < total; pass0 += (uint32_t)list_cap) {
        const uint32_t pass1 = min(total, pass0 + (uint32_t)list_cap);
        // an odd share keeps the threads' writes on different LDS banks
        const uint32_t share = ((pass1 - pass0 + kCandThreads - 1) / kCandThreads) | 1u;
        const uint32_t f_lo = pass0 + (uint32_t)tid * share;
        const uint32_t f_hi = min(pass1, f_lo + share);
        if (f_lo < f_hi) {
            int w = last_not_above(sp_pref, f_lo);  // the non-empty span that holds entry f_lo
            uint32_t base = sp_pref[w], ng = sp_pref[w + 1] - base;
            uint32_t where = sp_where[w], slen = sp_len[w];
            uint32_t k = f_lo - base;
            for (uint32_t f = f_lo; f < f_hi; ++f) {
                while (k >= ng) {  // next non-empty span (there is one: f < total)
                    ++w;
                    base = sp_pref[w];
                    ng = sp_pref[w + 1] - base;
                    where = sp_where[w];
                    slen = sp_len[w];
                    k = 0;
                }
                const int m = (int)(where & 3u);
                const int lo = max(m - (int)(4 * k), 0);
                const int hi = min(m + (int)slen - (int)(4 * k), 4);
                const uint32_t mask = ((1u << hi) - 1u) & ~((1u << lo) - 1u);
                list[f - pass0] = (((where >> 2) + k) << 4) | mask;
                ++k;
            }
        }
        __syncthreads();
        LSH_TRACE(3, 7);
        const int n = (int)(pass1 - pass0);
        for (int f0 = tid; f0 < n; f0 += kHitInFlight * kCandThreads) {
            uint32_t e[kHitInFlight];
            int4 x[kHitInFlight];
#pragma unroll
            for (int j = 0; j < kHitInFlight; ++j) {
                const int f = f0 + j * kCandThreads;
                e[j] = (f < n) ? list[f] : 0u;  // entry 0: group 0, nothing valid
            }
#pragma unroll
            for (int j = 0; j < kHitInFlight; ++j) x[j] = words4[e[j] >> 4];
#pragma unroll
            for (int j = 0; j < kHitInFlight; ++j) {
                bump(x[j].x, e[j] & 1u); bump(x[j].y, e[j] & 2u);
                bump(x[j].z, e[j] & 4u); bump(x[j].w, e[j] & 8u);
            }
        }
        LSH_TRACE(3, 4);
        __syncthreads();
    }
    LSH_TRACE(3, 5);
    // Eq. 10 for this row: bit j = (L[i, j] >= t).  Lane l of a wave reads counter word
    // 64 * c + l: its low half belongs to id 128 * c + 64 * (l / 32) + l % 32, its high half to
    // that id + 32, so the two ballots are four consecutive bitmap words (in the order
    // lo[31:0], hi[31:0], lo[63:32], hi[63:32]); lanes 0..3 store them.
    uint32_t* out = row_bitmaps + (size_t)r * nwords;
    const int w0 = id0 >> 5;                          // the slice's first bitmap word
    const int nchunks = (ncnt + kWave - 1) / kWave;   // counters of ids beyond V stay zero
    for (int c0 = wv; c0 < nchunks; c0 += 4 * kCandWaves) {  // four LDS reads in flight
        uint32_t x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = (c0 + q * kCandWaves) * kWave + ln;
            x[q] = (i < ncnt) ? cnt32[i] : 0u;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + q * kCandWaves;
            const uint64_t lo = __ballot((int)(x[q] & 0xFFFFu) >= t);
            const uint64_t hi = __ballot((int)(x[q] >> 16) >= t);
            const uint32_t mine = (ln == 0) ? (uint32_t)lo : (ln == 1) ? (uint32_t)hi
                                : (ln == 2) ? (uint32_t)(lo >> 32) : (uint32_t)(hi >> 32);
            if (ln < 4 && 4 * c + ln < ncnt / 16 && w0 + 4 * c + ln < nwords) out[w0 + 4 * c + ln] = mine;
        }
    }
    LSH_TRACE(3, 6);
}

// OR of B bitmaps of nwords words each (nwords apart) into the LDS bitmap bm; called by all
// kCandThreads threads, no barrier inside.
__device__ __forceinline__ void union_row_bitmaps(const uint32_t* __restrict__ rb, int B, int nwords,
                                                  uint32_t* bm) {
    for (int i = threadIdx.x; i < nwords; i += kCandThreads) {
        uint32_t x = 0;
        int b = 0;
        for (; b + 4 <= B; b += 4) {  // four independent loads in flight
            const uint32_t x0 = rb[(size_t)b * nwords + i], x1 = rb[(size_t)(b + 1) * nwords + i];
            const uint32_t x2 = rb[(size_t)(b + 2) * nwords + i], x3 = rb[(size_t)(b + 3) * nwords + i];
            x |= (x0 | x1) | (x2 | x3);
        }
        for (; b < B; ++b) x |= rb[(size_t)b * nwords + i];
        bm[i] = x;
    }
}

// grid = S workgroups: OR of the sentence's B row bitmaps and the top-frequent words, compacted.
__global__ void __launch_bounds__(kCandThreads)
k_union_compact(const uint32_t* __restrict__ row_bitmaps, int B, int V,
                const int32_t* __restrict__ topfreq, int T, int32_t* __restrict__ cand,
                int32_t* __restrict__ count) {
    extern __shared__ uint32_t smem[];  // union_compact_lds_words(V)
    const int s = blockIdx.x, tid = threadIdx.x;
    const int nwords = (V + 31) >> 5;
    uint32_t* bm = smem;
    uint32_t* wsum = smem + bitmap_words_padded(V);
    uint2* dlist = reinterpret_cast<uint2*>(wsum + 64);
    const int32_t tf_first = (tid < T) ? topfreq[tid] : -1;
    const int32_t tf_second = id_list_second(topfreq, T);
    union_row_bitmaps(row_bitmaps + (size_t)s * B * nwords, B, nwords, bm);
    __syncthreads();
    mark_id_list<true>(bm, V, topfreq, T, tf_first, tf_second);
    __syncthreads();
    compact_bitmap(bm, nwords, wsum, dlist, kUnionDenseCap, cand + (size_t)s * V, count + s);
}

}  // namespace lshbeam
