// Candidate generation fused into the logits kernel, for steps with little work (few sentences).
//
// With one sentence of a dozen beams the whole step moves ~9 MB: it is bound by its chain of
// dependent memory round trips and by kernel boundaries, not by bandwidth.  Here every workgroup
// of the logits grid rebuilds the sentence's presence bitmap for itself in LDS (hashing, cuckoo
// probes, bucket walk: ~70 KB of cache-resident reads), prefix-sums the bitmap words' popcounts,
// and finds the 16 candidates of each of its tiles by rank: a branch-free search of the prefix
// array for the word that holds the wanted output position, then the bit of that rank inside
// the word.  The candidate list is never needed before the contraction starts, so the separate
// candidates kernel, its compaction stores, and the count/list loads of the logits kernel all
// disappear; the dense ascending list is still emitted (each tile stores its 16 ids), because
// the selection kernel and the inspection calls read it.  The work is redundant across the
// workgroups on purpose: it runs concurrently on otherwise idle CUs and shortens the critical
// path.  Steps with many sentences keep the three-kernel path (there the candidates kernel is
// amortised and throughput matters, not latency).  With a hit threshold above 1, or with more
// beams than one chunk of hashing holds, the hashing stays in a kernel of its own and
// "rebuilding the bitmap" is the OR of the bitmaps that kernel left (k_union_logits).
//
// One launch per step: the log-softmax and the beam expansion run inside these kernels too.  The
// workgroups that had tiles of sentence s make their stores visible device-wide and take a ticket
// on a per-sentence counter; the one that draws the last ticket has everything it needs in
// memory and runs the selection (select.h) for the sentence -- no kernel boundary, no idle
// launch gap, no barrier across workgroups (nobody waits: a workgroup either finishes the
// sentence or exits).  The last arriver also puts the counter back to zero, so a captured graph
// can be replayed without clearing anything.  The tiles leave rich records (logits.h), from which
// the selection usually finishes without reading logits or candidate ids back.
#pragma once
#include "candidates.h"
#include "logits.h"
#include "select.h"

namespace lshbeam {

constexpr int kFusedWaves = kCandThreads / kWave;  // 16: the split-k width of the contraction

constexpr int kFusedRound = 16;                             // tiles of a workgroup looked up at a time
constexpr int kFusedTileIdWords = kFusedRound * kTileN;     // their candidate ids in LDS

// LDS words: candidate generation + the candidate ids of a round of tiles + the cross-wave
// reduction buffer of the contraction.
// (the selection of the one-launch plan reuses the same memory from its start: SelShared)
constexpr size_t kSelSharedWords = (sizeof(SelShared) + 3) / 4;
__host__ __device__ inline size_t fused_lds_words(int V, int P, int K, int stage_words) {
    const size_t need = candidates_lds_words(V, P, K, stage_words) + kFusedTileIdWords +
                        (size_t)kFusedWaves * 4 * kWave;
    return need > kSelSharedWords ? need : kSelSharedWords;
}

// Outputs and inputs of the step's tail (log-softmax + beam expansion) for the one-launch plan.
// (ONE_LAUNCH = false: the kernel stops after its tiles and a selection kernel follows.)
struct TailArgs {
    unsigned int* tickets;       // [S] counters, zero between steps
    const float* beam_scores;    // [S*B]
    float* lse;                  // [S*B]
    int32_t* out_beam;           // [S, B]
    int32_t* out_word;
    float* out_score;
    int tile_forced;             // 1..15: candidates per tile instead of 16 (option fused_tile)
};

// What follows the bitmap in both fused kernels.  Thread t owns a contiguous run of bitmap words;
// a workgroup scan of the runs' popcounts tells it which output positions of the ascending
// candidate list its set bits are.  The workgroup's tiles (g, g + G, ...) are taken kFusedRound at
// a time: every thread whose positions fall into one of them writes those ids to a small LDS
// table -- usually one or two threads per tile, walking at most 16 set bits -- and after a barrier
// the lanes of each tile read their candidate from it.  (Finding each lane's candidate by a
// search of a prefix array over all words -- a dozen dependent LDS reads per lane, behind a
// barrier that waited for the whole array -- cost a microsecond more.)
// `tile_ids` has kFusedRound * 16 words, `wsum` >= 17, `red` is the cross-wave reduction buffer;
// h_lds (or null) are the sentence's hidden rows staged in LDS as [B][d].
constexpr int kCoopBits = 8;   // list positions of one tile in one thread from which its wave shares the work
template <typename ET, bool ALIGNED, bool ONE_LAUNCH>
__device__ __forceinline__ void tiles_from_bitmap(const uint32_t* bm, uint32_t* wsum, uint32_t* tile_ids,
                                                  float (*red)[4][kWave], const float* h_lds,
                                                  const ET* __restrict__ E, int64_t ld, int d,
                                                  const float* __restrict__ H, int B, int V, int s,
                                                  int g, int G, int32_t* __restrict__ cand,
                                                  int32_t* __restrict__ count,
                                                  float* __restrict__ logits, int64_t cpitch,
                                                  TileRecords recs, const TailArgs& tail, uint32_t* smem) {
    const int tid = threadIdx.x, ln = lane_id();
    const int nwords = (V + 31) >> 5;
    const int per_thread = (nwords + kCandThreads - 1) / kCandThreads;
    const int wbeg = min(tid * per_thread, nwords), wend = min(wbeg + per_thread, nwords);
    uint32_t mine = 0;
    for (int i = wbeg; i < wend; ++i) mine += __popc(bm[i]);
    uint32_t total;
    const uint32_t run = block_incl_scan(mine, wsum, &total) - mine;   // first output position of my bits
    LSH_TRACE(0, 6);
    LSH_TRACE_WG(4);
    const int C = (int)total;

    const int tn = select_tile_width(C, tail.tile_forced, recs.pitch);
    const int ntiles = tn == kTileN ? (C + kTileN - 1) >> 4 : (C + tn - 1) / tn;   // (no division in the usual case)
    const int col = ln & 15;
    for (int base = 0; g + base * G < ntiles; base += kFusedRound) {
        // ids of the tiles g + (base + k) G, k < kFusedRound, into tile_ids[k][16].  A thread
        // with a few of a tile's positions walks its set bits itself.  One with kCoopBits or more
        // -- the dense words of the top-frequent ids put a whole tile into one thread, and sixteen
        // dependent steps of a single lane were the longest thing such a workgroup did -- hands
        // them to the lanes of its wave: lane c finds the c-th of them by rank (popcounts of the
        // owner's words, then a five-step search inside the word).
        for (int k = 0; k < kFusedRound; ++k) {
            const int nt = g + (base + k) * G;
            if (nt >= ntiles) break;
            const uint32_t lo = max(run, (uint32_t)(nt * tn));
            const uint32_t hi = min(min(run + mine, (uint32_t)(nt * tn + tn)), (uint32_t)C);
            const uint32_t n = (mine && lo < hi) ? hi - lo : 0u;
            uint32_t* ids_k = tile_ids + k * kTileN;             // [position in the list - t0]
            const uint32_t t0 = (uint32_t)(nt * tn);
            if (n > 0 && n < (uint32_t)kCoopBits) {
                // my (lo - run)-th set bit and the n - 1 that follow
                uint32_t skip = lo - run;
                int i = wbeg;
                uint32_t bits = bm[i];
                for (uint32_t c = __popc(bits); skip >= c; c = __popc(bits)) { skip -= c; bits = bm[++i]; }
                for (; skip; --skip) bits &= bits - 1u;
                for (uint32_t pos = lo; pos < hi; ++pos) {
                    while (!bits) bits = bm[++i];
                    ids_k[pos - t0] = ((uint32_t)i << 5) + (uint32_t)(__ffs(bits) - 1);
                    bits &= bits - 1u;
                }
            }
            for (uint64_t heavy = __ballot(n >= (uint32_t)kCoopBits); heavy; heavy &= heavy - 1) {   // (uniform)
                const int o = __ffsll((unsigned long long)heavy) - 1;
                const uint32_t o_lo = wave_read_lane(lo, o), o_n = wave_read_lane(n, o), o_run = wave_read_lane(run, o);
                int i = (int)wave_read_lane((uint32_t)wbeg, o);
                if ((uint32_t)ln < o_n) {
                    uint32_t r = o_lo - o_run + (uint32_t)ln;          // my bit's rank in the owner's words
                    uint32_t bits = bm[i];
                    for (uint32_t c = __popc(bits); r >= c; c = __popc(bits)) { r -= c; bits = bm[++i]; }
                    ids_k[o_lo + (uint32_t)ln - t0] = ((uint32_t)i << 5) + nth_set_bit(bits, r);
                }
            }
        }
        __syncthreads();
        for (int k = 0; k < kFusedRound; ++k) {
            const int nt = g + (base + k) * G;
            if (nt >= ntiles) break;
            // this lane's candidate: output position 16 nt + col of the ascending list (lanes past
            // the end of the list take the tile's first candidate; such columns are never stored)
            const bool in_list = col < tn && nt * tn + col < C;
            const int32_t id = (int32_t)tile_ids[k * kTileN + (in_list ? col : 0)];
            if (tid < kTileN && in_list)
                store_shared_result<ONE_LAUNCH>(&cand[(size_t)s * V + nt * tn + col], id);
            LSH_TRACE(1, 2);
            logits_tile_all_rows<ET, kFusedWaves, 64 / kFusedWaves, ALIGNED, 0, true, ONE_LAUNCH>(
                E, ld, d, H, B, s, nt, C, (int64_t)id, logits, cpitch, recs, red, h_lds, 0, 0, -1, tn);
        }
        // (a tile ends with a barrier: the table is free for the next round)
    }
    // (after the tiles: a barrier waits for the stores issued before it)
    if (g == 0 && tid == 0) store_shared_result<ONE_LAUNCH>(&count[s], (int32_t)C);
    if constexpr (!ONE_LAUNCH) return;

    // ---- the step's tail, by the last workgroup of the sentence to get here ----
    SelShared& sh = *reinterpret_cast<SelShared*>(smem);   // (bitmap, prefix, stage: all done with)
    const int participants = min(G, ntiles);               // workgroups of this sentence with tiles
    if (ntiles > 0) {
        if (g >= ntiles) return;
        // what the finishing workgroup reads of this one (logits, records, ids) went through to
        // memory (store_shared_result): once every wave's stores have completed, the ticket
        LSH_TRACE_LATEST(1, 12);
        publish_wait();
        __syncthreads();
        LSH_TRACE_LATEST(1, 13);
        if (tid == 0) {
            const unsigned int prev = atomicAdd(tail.tickets + s, 1u);
            const bool last = prev + 1u == (unsigned int)participants;
            if (last) atomicExch(tail.tickets + s, 0u);     // ready for the next step / replay
            sh.misc[7] = last ? 1u : 0u;
        }
        __syncthreads();
        if (sh.misc[7] == 0u) return;
        LSH_TRACE_ANY(1, 14);
    } else if (g != 0) {
        return;                // an empty list: workgroup 0 of the sentence pads the outputs
    }
    select_sentence<true, true>(sh, s, logits, cpitch, recs.rec, recs.id2, recs.pitch, cand, nullptr, C, V, B,
                          tail.beam_scores, tail.lse, tail.out_beam, tail.out_word, tail.out_score,
                          tail.tile_forced);
}

// grid = S * G workgroups: workgroup b works for sentence b % S and takes that sentence's tiles
// (b / S), (b / S) + G, ...
template <typename ET, bool ALIGNED, bool ONE_LAUNCH>
__global__ void __launch_bounds__(kCandThreads)
k_cand_logits(CandArgs a, const ET* __restrict__ E, int64_t ld, int S, int32_t* __restrict__ cand,
              int32_t* __restrict__ count, float* __restrict__ logits, int64_t cpitch,
              TileRecords recs, TailArgs tail) {
    extern __shared__ uint32_t smem[];
    // (one sentence, the usual case of this plan: no division before the first loads)
    const int s = S == 1 ? 0 : blockIdx.x % S;
    const int g = S == 1 ? blockIdx.x : blockIdx.x / S, G = S == 1 ? gridDim.x : gridDim.x / S;
    const int V = a.V, B = a.B;
    uint32_t* bm = smem;
    uint32_t* wsum = smem + candidates_lds_words(V, a.P, a.K, a.stage_words) - 64;
    uint32_t* tile_ids = smem + candidates_lds_words(V, a.P, a.K, a.stage_words);
    float (*red)[4][kWave] = reinterpret_cast<float (*)[4][kWave]>(tile_ids + kFusedTileIdWords);

    build_presence_bitmap(a, s, smem);
    // when the whole sentence was hashed in one chunk its hidden rows are still staged in LDS:
    // the contraction takes its A operands from there instead of reading H again
    const float* h_lds = nullptr;
    if (a.rows_chunk >= B && (a.d & 3) == 0)
        h_lds = reinterpret_cast<const float*>(smem + bitmap_words_padded(V));
    tiles_from_bitmap<ET, ALIGNED, ONE_LAUNCH>(bm, wsum, tile_ids, red, h_lds, E, ld, a.d, a.H, B, V, s, g, G, cand,
                                   count, logits, cpitch, recs, tail, smem);
    LSH_TRACE_WG(6);
}

// The same with the hashing done by an earlier kernel: the sentence's bitmap is the union of
// `nparts` bitmaps left in global memory (one per hidden row by k_hit_rows when the hit
// threshold is above 1, one per part of the sentence by k_part_bitmaps when it has many beams)
// and the top-frequent words (Eq. 3).
__host__ __device__ inline size_t union_logits_lds_words(int V) {
    const size_t need = (size_t)bitmap_words_padded(V) + 64 + kFusedTileIdWords +
                        (size_t)kFusedWaves * 4 * kWave;
    return need > kSelSharedWords ? need : kSelSharedWords;
}

template <typename ET, bool ALIGNED, bool ONE_LAUNCH>
__global__ void __launch_bounds__(kCandThreads)
k_union_logits(const uint32_t* __restrict__ part_bitmaps, int nparts, const int32_t* __restrict__ topfreq,
               int T, const ET* __restrict__ E, int64_t ld, int d, const float* __restrict__ H, int S,
               int B, int V, int32_t* __restrict__ cand, int32_t* __restrict__ count,
               float* __restrict__ logits, int64_t cpitch, TileRecords recs, TailArgs tail) {
    extern __shared__ uint32_t smem[];
    const int tid = threadIdx.x;
    const int s = blockIdx.x % S;
    const int g = blockIdx.x / S, G = gridDim.x / S;
    const int nwords = (V + 31) >> 5;
    uint32_t* bm = smem;
    uint32_t* wsum = bm + bitmap_words_padded(V);
    uint32_t* tile_ids = wsum + 64;
    float (*red)[4][kWave] = reinterpret_cast<float (*)[4][kWave]>(tile_ids + kFusedTileIdWords);

    const int32_t tf_first = (tid < T) ? topfreq[tid] : -1;
    union_row_bitmaps(part_bitmaps + (size_t)s * nparts * nwords, nparts, nwords, bm);
    __syncthreads();
    mark_id_list(bm, V, topfreq, T, tf_first);
    __syncthreads();
    tiles_from_bitmap<ET, ALIGNED, ONE_LAUNCH>(bm, wsum, tile_ids, red, nullptr, E, ld, d, H, B, V, s, g, G, cand,
                                   count, logits, cpitch, recs, tail, smem);
}

}  // namespace lshbeam
