// Gathered contraction  Logit[r, c] = sum_k H[r, k] * E[cand_s[c], k]   (Eq. 2 on the columns of
// the candidate list; the paper's separate "construct E_LSH" copy is fused away: candidate rows
// of E are gathered straight into the matrix-core operands).
//
// Besides the logits every tile leaves, per hidden row, the pair (max, sum exp(logit - max)) over
// its 16 candidates: the selection combines these into the row's log-sum-exp without touching the
// exponential of every logit again.  The fused kernels (fused.h) leave a richer record per row and
// tile (TileRecord): also the word id of the maximum, the second largest logit of the tile and
// its word id -- enough for the selection to finish, in the common case, without reading a
// single logit or candidate id back.
//
// Work unit ("tile"): one sentence s, one group of 16 hidden rows (M-tile) and 16 candidates.
// A workgroup of WAVES waves splits the hidden dimension between its waves; every wave issues
// v_mfma_f32_16x16x4_f32 over its share of k and the partial 16x16 tiles are summed through LDS
// in a fixed wave order (deterministic).
//
// Operand layout of v_mfma_f32_16x16x4_f32 (A is 16x4, B is 4x16, D is 16x16, 64 lanes):
//   lane l supplies A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16];
//   lane l receives D[i = 4 * (l / 16) + r][j = l % 16] in accumulator register r = 0..3.
// The k slots of one instruction may hold any four k indices as long as A and B agree, so lane l
// loads ONE 16-byte chunk of its candidate's row (fp32: 4 consecutive k, bf16: 8) and feeds one
// element per instruction: per load instruction a wave touches 16 rows x 64 contiguous bytes.
//
// Drivers of the tile code:
//   k_logits<WAVES>  a workgroup of 16 or 4 waves per (tile, row group), k split over the waves
//                    (few sentences; more than 64 beams);
//   k_logits_wave    one wave per tile, up to four row groups in the wave, hidden rows read from
//                    global memory (kept as the LSHBEAM_LOGITS_HLDS=0 path);
//   k_logits_hlds    one wave per tile, the sentence's hidden rows staged in LDS (up to 32 beams:
//                    the bandwidth-bound case; more beams in groups of 16 rows);
//   k_logits_estage  33..64 beams: hidden rows in registers, candidate rows through LDS;
//   fused.h          the same tiles inside the kernels that also produce the candidate list.
#pragma once
#include "candidates.h"
#include "device_utils.h"

namespace lshbeam {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <typename ET> struct ElemTraits;
template <> struct ElemTraits<float> {
    static constexpr int VEC = 4;  // elements per 16-byte load
    __device__ static __forceinline__ void load16(const float* p, float (&out)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
};
template <> struct ElemTraits<uint16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void load16(const uint16_t* p, float (&out)[8]) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

// Per (hidden row, tile) record of the fused kernels (the other kernels store the first two fields
// only, as a float2 array in the same place): x = largest logit of the tile's candidates,
// y = sum exp(logit - x), z = second largest logit (-inf if the tile has one candidate), w = word id
// of the largest (the lowest column among equals; as bits).  The id of the second largest goes to
// a parallel int32 array (-1 if none).  The plain kernels store only (x, y) as a float2.
typedef float4 TileRecord;
struct TileRecords {
    TileRecord* rec;   // [rows, pitch]
    int32_t* id2;      // [rows, pitch] word id of each record's second largest logit, -1 if none
    int64_t pitch;     // records per hidden row
};

// Records that stand for groups of tiles.  A kernel whose workgroup j of G walks the tiles j,
// j + G, j + 2G, ... of a sentence leaves one record for every kGroupTiles of them: record
// j + m G covers the tiles j + (kGroupTiles m + i) G, i < kGroupTiles.  (Fifty rows of per-tile
// records were 140 KB per sentence, all of which has to enter the one CU that selects.)
constexpr int kGroupTiles = 8;
__host__ __device__ inline int group_records(int ntiles, int G) {   // record slots per hidden row
    const int per_wg = (ntiles + G - 1) / G;
    return ntiles < G ? ntiles : G * ((per_wg + kGroupTiles - 1) / kGroupTiles);
}

constexpr int kTileN = 16;  // candidates per tile
constexpr int kTileM = 16;  // hidden rows per tile
constexpr int kMaxSentencesLogits = 4096;

// One (hidden row, tile) record from the 16 lanes that hold the row's logits of the tile's columns
// (a DPP row: 16 consecutive lanes, lane jc = column jc; `valid` lanes hold a logit x of a real
// candidate `id`).  Eq. 1 denominator, first stage: (max, sum of exp(logit - max)).  RICH (the
// fused kernels): plus the second largest logit and the two word ids, as a TileRecord; otherwise
// the pair alone, as a float2 in the same array (the contraction kernels of the many-tile plans
// are bound by bandwidth and instruction issue, and the longer epilogue cost them 4-8 %).
// Called by whole DPP rows; rows with row_ok false store nothing.  SHARE: see store_shared_result.
template <bool SHARE, bool RICH>
__device__ __forceinline__ void tile_record_store(const TileRecords& recs, size_t at, bool row_ok, bool valid,
                                                  float x, int jc, int32_t id) {
    const float mx = row16_max(valid ? x : -INFINITY);
    const float se = row16_sum(valid ? expf(x - mx) : 0.f);
    if constexpr (!RICH) {
        if (jc == 0 && row_ok) reinterpret_cast<float2*>(recs.rec)[at] = make_float2(mx, se);
    } else {
        // the lowest column that holds the maximum; the largest of the others and its lowest column
        const int c1 = row16_min_i32((valid && x == mx) ? jc : 16);
        const float mx2 = row16_max((valid && jc != c1) ? x : -INFINITY);
        const int c2 = row16_min_i32((valid && jc != c1 && x == mx2) ? jc : 16);
        if (row_ok) {
            if (jc == (c1 < 16 ? c1 : 0)) {   // (no column equals the maximum: NaN logits)
                unsigned long long* rec = reinterpret_cast<unsigned long long*>(recs.rec + at);
                const uint32_t idb = (uint32_t)(c1 < 16 ? id : -1);
                store_shared_result<SHARE>(rec, ((unsigned long long)__float_as_uint(se) << 32) | __float_as_uint(mx));
                store_shared_result<SHARE>(rec + 1, ((unsigned long long)idb << 32) | __float_as_uint(mx2));
            }
            if (jc == (c2 < 16 ? c2 : 0)) store_shared_result<SHARE>(&recs.id2[at], c2 < 16 ? id : (int32_t)-1);
        }
    }
}

// MTB tiles: logits of hidden rows [16 mt, 16 (mt + MTB)) of sentence s against 16 candidates,
// this lane's candidate being row j of E (lanes beyond the list hold any valid row; their results
// are dropped; row groups beyond B are computed on clamped rows and dropped too).  The candidate
// rows are loaded once for all MTB row groups.  Called by all WAVES*64 threads of the workgroup;
// contains 2 MTB workgroup barriers.  h_lds, if given, is an LDS copy of the sentence's B hidden
// rows (16-byte aligned, pitch h_pitch floats; 0 = d).  [row_lo, row_hi) restricts the call to
// a range of the sentence's rows (mt counts groups of 16 from row_lo; h_lds then holds that range).
//
// ALIGNED: E rows and H rows can be read with 16-byte vector loads (pointers 16-byte aligned,
// d and the pitches multiples of the vector width).  Otherwise elements are read one by one.
template <typename ET, int WAVES, int UNROLL, bool ALIGNED, int MTB = 1, bool RICH = false, bool SHARE = false>
__device__ __forceinline__ void logits_tile(const ET* __restrict__ E, int64_t ld, int d,
                                            const float* __restrict__ H, int B, int s, int mt,
                                            int nt, int C, int64_t j, float* __restrict__ logits,
                                            int64_t cpitch, TileRecords recs, float (*red)[4][kWave],
                                            const float* h_lds = nullptr, int h_pitch = 0,
                                            int row_lo = 0, int row_hi = -1, int tn = kTileN) {
    // tn <= 16: candidates of this tile (columns tn .. 15 of the matrix instruction stay unused;
    // narrower tiles are an option of the fused plans, see select_tile_width)
    constexpr int VEC = ElemTraits<ET>::VEC;
    constexpr int KSTEP = 4 * VEC;  // k covered by one 64-lane load
    if (h_pitch == 0) h_pitch = d;
    if (row_hi < 0) row_hi = B;
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    const int col = ln & 15, kq = ln >> 4;
    const int nks = (d + KSTEP - 1) / KSTEP;
    const int n0 = nt * tn;
    const bool col_used = col < tn;   // lanes of unused columns load no candidate row
    const ET* erow = E + j * ld;
    // the sentence's hidden rows, from LDS when the caller has them staged there ([B][d]);
    // rows beyond B are clamped like the candidate: never stored
    const float* hrow[MTB];
#pragma unroll
    for (int m = 0; m < MTB; ++m) {
        const int hr = min(row_lo + (mt + m) * kTileM + col, row_hi - 1);
        hrow[m] = h_lds ? h_lds + (size_t)(hr - row_lo) * h_pitch : H + ((size_t)s * B + hr) * d;
    }

    floatx4 acc[MTB];
#pragma unroll
    for (int m = 0; m < MTB; ++m) acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int ks0 = wv; ks0 < nks; ks0 += WAVES * UNROLL) {
        float ev[UNROLL][VEC], hv[MTB][UNROLL][VEC];
#pragma unroll
        for (int uu = 0; uu < UNROLL; ++uu) {
            const int k = (ks0 + uu * WAVES) * KSTEP + kq * VEC;
            if (ALIGNED) {
                if (k < d) {
                    if (col_used) {
                        ElemTraits<ET>::load16(erow + k, ev[uu]);
                    } else {
#pragma unroll
                        for (int q = 0; q < VEC; ++q) ev[uu][q] = 0.f;
                    }
#pragma unroll
                    for (int m = 0; m < MTB; ++m)
#pragma unroll
                        for (int q = 0; q < VEC; q += 4) {
                            const float4 h4 = *reinterpret_cast<const float4*>(hrow[m] + k + q);
                            hv[m][uu][q] = h4.x; hv[m][uu][q + 1] = h4.y;
                            hv[m][uu][q + 2] = h4.z; hv[m][uu][q + 3] = h4.w;
                        }
                } else {
#pragma unroll
                    for (int q = 0; q < VEC; ++q) {
                        ev[uu][q] = 0.f;
#pragma unroll
                        for (int m = 0; m < MTB; ++m) hv[m][uu][q] = 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int q = 0; q < VEC; ++q) {
                    const bool in = (k + q) < d;
                    ev[uu][q] = (in && col_used) ? elem_f32(erow + k + q) : 0.f;
#pragma unroll
                    for (int m = 0; m < MTB; ++m) hv[m][uu][q] = in ? hrow[m][k + q] : 0.f;
                }
            }
        }
#pragma unroll
        for (int uu = 0; uu < UNROLL; ++uu)
#pragma unroll
            for (int q = 0; q < VEC; ++q)
#pragma unroll
                for (int m = 0; m < MTB; ++m)
                    acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[m][uu][q], ev[uu][q], acc[m],
                                                                  0, 0, 0);
    }

    LSH_TRACE(1, 3);
    LSH_TRACE_WG(5);
#pragma unroll
    for (int m = 0; m < MTB; ++m) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wv][r][ln] = acc[m][r];
        __syncthreads();
        LSH_TRACE_WG(7);
        if (tid < kTileM * kTileN) {
            const int i = tid >> 4, jc = tid & 15;
            const int src = (i >> 2) * 16 + jc, r = i & 3;
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) sum += red[w][r][src];
            const int row = row_lo + (mt + m) * kTileM + i, c = n0 + jc;
            const bool valid = row < row_hi && jc < tn && c < C;
            // (SHARE: other workgroups of this kernel read the results; see store_shared_result)
            if (valid) store_shared_result<SHARE>(&logits[((size_t)s * B + row) * cpitch + c], sum);
            tile_record_store<SHARE, RICH>(recs, ((size_t)s * B + row) * recs.pitch + nt, row < row_hi, valid, sum,
                                           jc, (int32_t)j);
        }
        __syncthreads();
    }
    LSH_TRACE(1, 4);
}

// All row groups of one tile of candidates, the candidate rows being read once for up to four
// groups (64 beams) at a time.
template <typename ET, int WAVES, int UNROLL, bool ALIGNED, int FIXED_MT = 0, bool RICH = false, bool SHARE = false>
__device__ __forceinline__ void logits_tile_all_rows(const ET* __restrict__ E, int64_t ld, int d,
                                                     const float* __restrict__ H, int B, int s,
                                                     int nt, int C, int64_t j,
                                                     float* __restrict__ logits, int64_t cpitch,
                                                     TileRecords recs, float (*red)[4][kWave],
                                                     const float* h_lds = nullptr, int h_pitch = 0,
                                                     int row_lo = 0, int row_hi = -1, int tn = kTileN) {
    // loads in flight per row group shrink as the groups grow: the operands of all groups have
    // to fit the register budget of a 1024-thread workgroup
    // (measured: keeping the full unroll in 256-thread workgroups, where registers would allow
    // it, is slower -- the hidden-row loads of four groups then crowd out the candidate rows)
    constexpr int U4 = UNROLL >= 4 ? UNROLL / 4 : 1;
    constexpr int U2 = ElemTraits<ET>::VEC > 4 ? U4 : (UNROLL >= 2 ? UNROLL / 2 : 1);
    // FIXED_MT: the caller knows the number of row groups at compile time (only that case is
    // instantiated, so its registers do not count against the others)
    const int MT = FIXED_MT ? FIXED_MT : ((row_hi < 0 ? B : row_hi - row_lo) + kTileM - 1) / kTileM;
    if (MT == 1) {
        logits_tile<ET, WAVES, UNROLL, ALIGNED, 1, RICH, SHARE>(E, ld, d, H, B, s, 0, nt, C, j, logits, cpitch,
            recs, red, h_lds, h_pitch, row_lo, row_hi, tn);
    } else if (MT == 2) {
        logits_tile<ET, WAVES, U2, ALIGNED, 2, RICH, SHARE>(E, ld, d, H, B, s, 0, nt, C, j, logits, cpitch,
            recs, red, h_lds, h_pitch, row_lo, row_hi, tn);
    } else if (ElemTraits<ET>::VEC > 4) {  // bf16: twice the registers per load, two groups at most
        for (int mt = 0; mt < MT; mt += 2)
            logits_tile<ET, WAVES, U2, ALIGNED, 2, RICH, SHARE>(E, ld, d, H, B, s, mt, nt, C, j, logits, cpitch,
            recs, red, h_lds, h_pitch, row_lo, row_hi, tn);
    } else {
        for (int mt = 0; mt < MT; mt += 4)
            logits_tile<ET, WAVES, U4, ALIGNED, 4, RICH, SHARE>(E, ld, d, H, B, s, mt, nt, C, j, logits, cpitch,
            recs, red, h_lds, h_pitch, row_lo, row_hi, tn);
    }
}

template <typename ET, int WAVES, int UNROLL, bool ALIGNED>
__global__ void __launch_bounds__(WAVES * kWave)
k_logits(const ET* __restrict__ E, int64_t ld, int d, const float* __restrict__ H, int S, int B,
         const int32_t* __restrict__ cand, const int32_t* __restrict__ count, int V,
         float* __restrict__ logits, int64_t cpitch, TileRecords recs) {
    __shared__ uint32_t tile_pref[kMaxSentencesLogits + 1];
    __shared__ float red[WAVES][4][kWave];

    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    (void)tid;
    const int MT = (B + kTileM - 1) / kTileM;

    LSH_TRACE(1, 0);
    // Workgroups are dealt to the 8 XCDs round-robin by the dispatcher; renumber them so that
    // consecutive logical ids (which take neighbouring tiles) share an XCD and its L2.
    // (Only worth it when several M-tiles re-read the same candidate rows; with one M-tile the
    // plain order lets the first workgroups dispatched be the ones that have work.)
    const uint32_t G = gridDim.x;
    const uint32_t per_xcd = G >> 3;
    const uint32_t logical = ((G & 7u) || MT == 1) ? blockIdx.x
                                                   : (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    const int col = ln & 15;

    // With a single sentence the first tile's candidate ids do not depend on the count: request
    // them together with it instead of after it (one dependent memory round trip less).
    const bool spec = (S == 1) && (cand != nullptr);
    int32_t jspec = 0;
    if (spec) {
        const uint32_t c0 = (logical / (uint32_t)MT) * kTileN + col;
        if (c0 < (uint32_t)V) jspec = cand[c0];
    }

    // exclusive prefix of tiles per sentence (wave 0, 64 sentences at a time)
    if (wv == 0) {
        uint32_t carry = 0;
        for (int base = 0; base < S; base += kWave) {
            const int s = base + ln;
            uint32_t n = 0;
            if (s < S) {
                const int C = count ? count[s] : V;
                n = (uint32_t)MT * (uint32_t)((C + kTileN - 1) / kTileN);
            }
            const uint32_t incl = wave_incl_scan(n);
            if (s < S) tile_pref[s] = carry + incl - n;
            carry += wave_read_lane(incl, kWave - 1);
        }
        if (ln == 0) tile_pref[S] = carry;
    }
    __syncthreads();
    LSH_TRACE(1, 1);
    const uint32_t total_tiles = tile_pref[S];

    for (uint32_t t = logical; t < total_tiles; t += G) {
        int lo = 0, hi = S;  // sentence: last s with tile_pref[s] <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tile_pref[mid] <= t) lo = mid; else hi = mid;
        }
        const int s = lo;
        const uint32_t tl = t - tile_pref[s];
        const int nt = tl / MT, mt = tl - nt * MT;
        const int C = count ? count[s] : V;
        const int n0 = nt * kTileN;

        // out-of-range lanes are clamped onto a valid row; their results are never stored
        const int cidx = min(n0 + col, C - 1);
        int64_t j;
        if (spec && t == logical)  // column 0 of a tile is always a real candidate
            j = (n0 + col < C) ? jspec : __shfl(jspec, ln & ~15, kWave);
        else
            j = cand ? cand[(size_t)s * V + cidx] : cidx;
        LSH_TRACE(1, 2);
        logits_tile<ET, WAVES, UNROLL, ALIGNED>(E, ld, d, H, B, s, mt, nt, C, j, logits, cpitch, recs, red);
    }
}

// Throughput variant for steps with many tiles (many sentences): ONE WAVE per tile of 16
// candidates, all k and all MT groups of 16 hidden rows in that wave.  No LDS, no barrier: the
// accumulators go straight from the matrix core to the stores, and a candidate row is read once
// however many beams there are.  Waves of a workgroup take consecutive tiles; the grid is
// persistent.
//
// Whole rounds (every wave of the grid one tile) run this way.  A last (or only) round that would
// occupy fewer than half of the waves is different: while all waves stream, the kernel runs at the
// memory system's rate, but a few hundred waves left alone with a 64 KB tile each run at one
// wave's latency-bound rate, and that tail was a sixth of the kernel.  Such a remainder is
// therefore dealt to whole workgroups, whose four waves split k and sum their partial tiles
// through LDS in wave order (logits_tile): four times as many waves share the same bytes.
template <typename ET, int MT, int UNROLL, bool ALIGNED>
__global__ void __launch_bounds__(256)
k_logits_wave(const ET* __restrict__ E, int64_t ld, int d, const float* __restrict__ H, int S, int B,
              const int32_t* __restrict__ cand, const int32_t* __restrict__ count, int V,
              float* __restrict__ logits, int64_t cpitch, TileRecords recs) {
    constexpr int VEC = ElemTraits<ET>::VEC;
    constexpr int KSTEP = 4 * VEC;
    __shared__ uint32_t tile_pref[kMaxSentencesLogits + 1];
    __shared__ float red[4][4][kWave];
    const int ln = lane_id(), wv = wave_id();
    LSH_TRACE(1, 0);
    if (wv == 0) {
        uint32_t carry = 0;
        for (int base = 0; base < S; base += kWave) {
            const int s = base + ln;
            uint32_t n = 0;
            if (s < S) n = (uint32_t)(((count ? count[s] : V) + kTileN - 1) / kTileN);
            const uint32_t incl = wave_incl_scan(n);
            if (s < S) tile_pref[s] = carry + incl - n;
            carry += wave_read_lane(incl, kWave - 1);
        }
        if (ln == 0) tile_pref[S] = carry;
    }
    __syncthreads();
    LSH_TRACE(1, 1);
    const uint32_t total_tiles = tile_pref[S];
    const uint32_t nwaves = gridDim.x * 4u;
    const int col = ln & 15, kq = ln >> 4;
    const int nks = (d + KSTEP - 1) / KSTEP;
    // tiles [0, wave_tiles) one wave each; the rest one workgroup each
    const uint32_t whole = total_tiles / nwaves * nwaves;
    const uint32_t wave_tiles = ((total_tiles - whole) * 2u > nwaves) ? total_tiles : whole;
    auto sentence_of = [&](uint32_t t) {
        int lo = 0, hi = S;  // last s with tile_pref[s] <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tile_pref[mid] <= t) lo = mid; else hi = mid;
        }
        return lo;
    };

    // workgroup b takes the consecutive tiles [b * per_wg, (b + 1) * per_wg), dealt round-robin to
    // its waves: neighbouring tiles (same sentence, same hidden rows in L1) stay together, and
    // with fewer tiles than waves every workgroup (hence every CU) still gets its share
    const uint32_t per_wg = (wave_tiles + gridDim.x - 1) / gridDim.x;
    const uint32_t wg_end = min(wave_tiles, (blockIdx.x + 1u) * per_wg);
    for (uint32_t t = blockIdx.x * per_wg + wv; t < wg_end; t += 4u) {
        const int s = sentence_of(t);
        const int nt = (int)(t - tile_pref[s]);
        const int C = count ? count[s] : V;
        const int n0 = nt * kTileN;
        const int cidx = min(n0 + col, C - 1);  // clamped lanes are never stored
        const int64_t j = cand ? cand[(size_t)s * V + cidx] : cidx;
        const ET* erow = E + j * ld;
        const float* hrow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            hrow[mt] = H + ((size_t)s * B + min(mt * kTileM + col, B - 1)) * d;

        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int ks0 = 0; ks0 < nks; ks0 += UNROLL) {
            float ev[UNROLL][VEC], hv[MT][UNROLL][VEC];
#pragma unroll
            for (int uu = 0; uu < UNROLL; ++uu) {
                const int k = (ks0 + uu) * KSTEP + kq * VEC;
                if (ALIGNED) {
                    if (k < d) {
                        ElemTraits<ET>::load16(erow + k, ev[uu]);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int q = 0; q < VEC; q += 4) {
                                const float4 h4 = *reinterpret_cast<const float4*>(hrow[mt] + k + q);
                                hv[mt][uu][q] = h4.x; hv[mt][uu][q + 1] = h4.y;
                                hv[mt][uu][q + 2] = h4.z; hv[mt][uu][q + 3] = h4.w;
                            }
                    } else {
#pragma unroll
                        for (int q = 0; q < VEC; ++q) {
                            ev[uu][q] = 0.f;
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt) hv[mt][uu][q] = 0.f;
                        }
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < VEC; ++q) {
                        const bool in = (k + q) < d;
                        ev[uu][q] = in ? elem_f32(erow + k + q) : 0.f;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) hv[mt][uu][q] = in ? hrow[mt][k + q] : 0.f;
                    }
                }
            }
#pragma unroll
            for (int uu = 0; uu < UNROLL; ++uu)
#pragma unroll
                for (int q = 0; q < VEC; ++q)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[mt][uu][q], ev[uu][q],
                                                                       acc[mt], 0, 0, 0);
        }
        // lane (col, kq) holds rows 16 mt + 4 kq + r of column n0 + col: 16 lanes per row
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = mt * kTileM + 4 * kq + r, c = n0 + col;
                const bool valid = row < B && c < C;
                const float x = acc[mt][r];
                if (valid) logits[((size_t)s * B + row) * cpitch + c] = x;
                tile_record_store<false, false>(recs, ((size_t)s * B + row) * recs.pitch + nt, row < B, valid, x, col,
                                         (int32_t)j);
            }
    }

    // the remainder: one workgroup per tile, k split over its four waves (uniform per workgroup)
    for (uint32_t t = wave_tiles + blockIdx.x; t < total_tiles; t += gridDim.x) {
        const int s = sentence_of(t);
        const int nt = (int)(t - tile_pref[s]);
        const int C = count ? count[s] : V;
        const int cidx = min(nt * kTileN + col, C - 1);
        const int64_t j = cand ? cand[(size_t)s * V + cidx] : cidx;
        logits_tile_all_rows<ET, 4, (UNROLL < 4 ? UNROLL : 4), ALIGNED, MT>(E, ld, d, H, B, s, nt, C, j,
                                                                        logits, cpitch, recs, red);
    }
}

// The wave-per-tile kernel with the hidden rows in LDS.  Measured on this machine: a stream of
// 16-byte loads that hits in cache still costs as much load-path throughput as one that goes to
// memory -- gathering candidate rows alone runs at 6.7 TB/s, with an equal stream of hidden-row
// loads beside it at 3.4 TB/s.  The A operands therefore must not come through the vector memory
// path at all: a workgroup (WAVES waves, consecutive tiles, so mostly one sentence) stages the
// sentence's hidden rows in LDS once and every tile reads them with ds_read_b128.  More rows
// than LDS holds are taken in groups, a workgroup each: every group reads the candidate rows
// again (the groups of a block of tiles run on one XCD, so from its L2 mostly), which is still far less load traffic than
// hidden rows coming through the vector memory path.  The row
// pitch is the next value >= d that is 4 modulo 32: consecutive rows then start 4 banks apart
// and eight lanes x 16 bytes (eight rows, same k) cover all 32 banks exactly once.
__host__ __device__ inline int hlds_pitch(int d) {
    int p = (d + 3) & ~3;
    while (p % 32 != 4) p += 4;
    return p;
}
// bf16 candidate rows with 16-byte aligned operands: the hidden rows are staged as three bf16
// planes hi + mid + lo = h exactly (8 + 8 + 8 significand bits: each plane is the remainder so
// far truncated to bf16), and the contraction runs on v_mfma_f32_16x16x32_bf16 -- a lane's
// 16-byte chunk of its candidate row IS that instruction's B operand (8 consecutive k), no
// widening; three instructions per chunk against eight fp32 ones at a quarter of the cycles each.
// Products of two bf16 values are exact in fp32, so the result differs from the widened fp32
// contraction by summation order only.  Plane rows are pitched 8 modulo 64 elements (16 modulo
// 128 bytes: eight rows x 16 bytes cover all banks once).
__host__ __device__ inline int hlds_pitch_planes(int d) {
    int p = (d + 7) & ~7;
    while (p % 64 != 8) p += 8;
    return p;
}
// dynamic LDS: tile prefix (S + 1 words, rounded to 4), split-k reduction buffer, hidden rows
// (fp32, or three bf16 planes)
__host__ __device__ inline size_t hlds_lds_bytes(int S, int rows, int d, int waves, bool planes = false) {
    const size_t hidden = planes ? (size_t)rows * hlds_pitch_planes(d) * 6 : (size_t)rows * hlds_pitch(d) * 4;
    return ((size_t)((S + 1 + 3) & ~3) + (size_t)waves * 4 * kWave) * 4 + hidden;
}
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename ET, int MT, int WAVES, int UNROLL, bool ALIGNED, bool PLANES = false>
__global__ void __launch_bounds__(WAVES * kWave) __attribute__((amdgpu_waves_per_eu(4)))
k_logits_hlds(const ET* __restrict__ E, int64_t ld, int d, const float* __restrict__ H, int S, int B,
              int group_rows /*row group g takes rows [g, g + 1) * group_rows of every sentence;
                               group_rows <= 16 MT*/,
              int gx /*workgroups per row group*/, int ngroups, int rem_div,
              const int32_t* __restrict__ cand, const int32_t* __restrict__ count, int V,
              float* __restrict__ logits, int64_t cpitch, TileRecords recs) {
    constexpr int VEC = ElemTraits<ET>::VEC;
    constexpr int KSTEP = 4 * VEC;
    extern __shared__ uint32_t hsm[];
    // grid = round_up(gx, 8) * ngroups workgroups.  Workgroup ids go round the 8 XCDs, and the
    // row groups that read the same candidate rows should share an L2: ids that are congruent
    // modulo 8 and consecutive otherwise form the row groups of one block of tiles.
    const uint32_t wg_slot = blockIdx.x >> 3;
    const uint32_t bx = (wg_slot / (uint32_t)ngroups) * 8u + (blockIdx.x & 7u);
    const int by = (int)(wg_slot % (uint32_t)ngroups);
    if (bx >= (uint32_t)gx) return;
    const int row0 = by * group_rows, Bg = min(group_rows, B - row0);
    uint32_t* tile_pref = hsm;
    float (*red)[4][kWave] = reinterpret_cast<float (*)[4][kWave]>(hsm + ((S + 1 + 3) & ~3));
    float* hl = reinterpret_cast<float*>(hsm + ((S + 1 + 3) & ~3) + WAVES * 4 * kWave);
    const int pitch = hlds_pitch(d);
    // PLANES (bf16 rows, ALIGNED): hidden rows as three bf16 planes, bf16 matrix instructions
    static_assert(!PLANES || (ALIGNED && VEC == 8), "bf16 planes need aligned bf16 rows");
    const int ppitch_h = hlds_pitch_planes(d);
    uint16_t* hplane = reinterpret_cast<uint16_t*>(hl);
    const size_t plane_stride = (size_t)group_rows * ppitch_h;
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    LSH_TRACE(1, 0);
    if (wv == 0) {
        uint32_t carry = 0;
        for (int base = 0; base < S; base += kWave) {
            const int s = base + ln;
            uint32_t n = 0;
            if (s < S) n = (uint32_t)(((count ? count[s] : V) + kTileN - 1) / kTileN);
            const uint32_t incl = wave_incl_scan(n);
            if (s < S) tile_pref[s] = carry + incl - n;
            carry += wave_read_lane(incl, kWave - 1);
        }
        if (ln == 0) tile_pref[S] = carry;
    }
    __syncthreads();
    LSH_TRACE(1, 1);
    const uint32_t total_tiles = tile_pref[S];
    const uint32_t nwaves = (uint32_t)gx * (uint32_t)WAVES;
    const int col = ln & 15, kq = ln >> 4;
    const int nks = (d + KSTEP - 1) / KSTEP;
    const uint32_t whole = total_tiles / nwaves * nwaves;
    // a last round that fills at most 1 / rem_div of the waves is dealt to whole workgroups that
    // split k (below); a fuller one runs as one more wave-per-tile round (measured with rem_div = 4
    // against 2: S = 32, B = 20: 117 -> 83 us; the 64-sentence bf16 shape: 229 -> 221 us)
    const uint32_t wave_tiles = ((total_tiles - whole) * (uint32_t)rem_div > nwaves) ? total_tiles : whole;
    auto sentence_of = [&](uint32_t t) {
        int lo = 0, hi = S;  // last s with tile_pref[s] <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tile_pref[mid] <= t) lo = mid; else hi = mid;
        }
        return lo;
    };
    int staged = -1;
    auto stage = [&](int s) {  // workgroup-uniform; barriers inside
        if (s == staged) return;
        __syncthreads();  // everyone is done with the previous sentence's rows
        const float* Hs = H + ((size_t)s * B + row0) * d;
        if constexpr (PLANES) {  // (ALIGNED: d is a multiple of 8 and H is 16-byte aligned)
            const int d4 = d >> 2;
            for (int e = tid; e < Bg * d4; e += WAVES * kWave) {
                const int r = e / d4, c = e - r * d4;
                const float4 v = reinterpret_cast<const float4*>(Hs)[e];
                const float x[4] = {v.x, v.y, v.z, v.w};
                uint32_t pl[3][4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t hi = __float_as_uint(x[q]) & 0xFFFF0000u;
                    const float r1 = x[q] - __uint_as_float(hi);          // exact
                    const uint32_t mid = __float_as_uint(r1) & 0xFFFF0000u;
                    const float r2 = r1 - __uint_as_float(mid);           // exact, <= 8 bits
                    pl[0][q] = hi >> 16; pl[1][q] = mid >> 16; pl[2][q] = __float_as_uint(r2) >> 16;
                }
#pragma unroll
                for (int pnum = 0; pnum < 3; ++pnum)
                    *reinterpret_cast<uint2*>(hplane + pnum * plane_stride + (size_t)r * ppitch_h + 4 * c) =
                        make_uint2(pl[pnum][0] | (pl[pnum][1] << 16), pl[pnum][2] | (pl[pnum][3] << 16));
            }
        } else if ((d & 3) == 0 && ((uintptr_t)Hs & 15) == 0) {
            const int d4 = d >> 2;
            for (int e = tid; e < Bg * d4; e += WAVES * kWave) {
                const int r = e / d4, c = e - r * d4;
                *reinterpret_cast<float4*>(hl + (size_t)r * pitch + 4 * c) =
                    reinterpret_cast<const float4*>(Hs)[e];
            }
        } else {
            for (int e = tid; e < Bg * d; e += WAVES * kWave) {
                const int r = e / d, c = e - r * d;
                hl[(size_t)r * pitch + c] = Hs[e];
            }
        }
        __syncthreads();
        staged = s;
    };

    // whole rounds: one wave per tile; the workgroup walks its consecutive tiles sentence by
    // sentence (all of its waves in the same sentence, so one staging serves them)
    const uint32_t per_wg = (wave_tiles + (uint32_t)gx - 1) / (uint32_t)gx;
    const uint32_t wg_begin = min(wave_tiles, bx * per_wg);
    const uint32_t wg_end = min(wave_tiles, wg_begin + per_wg);
    for (uint32_t seg = wg_begin; seg < wg_end;) {
        const int s = sentence_of(seg);
        const uint32_t seg_end = min(wg_end, tile_pref[s + 1]);
        stage(s);
        LSH_TRACE(1, 2);
        const int C = count ? count[s] : V;
        for (uint32_t t = seg + wv; t < seg_end; t += WAVES) {
            const int nt = (int)(t - tile_pref[s]);
            const int n0 = nt * kTileN;
            const int cidx = min(n0 + col, C - 1);  // clamped lanes are never stored
            const int64_t j = cand ? cand[(size_t)s * V + cidx] : cidx;
            const ET* erow = E + j * ld;
            const float* hrow[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) hrow[mt] = hl + (size_t)min(mt * kTileM + col, Bg - 1) * pitch;
            floatx4 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
            if constexpr (PLANES) {
                // the rolling prefetch of the branch below, on raw 16-byte chunks (half the
                // registers of the widened form, so twice the loads in flight)
                constexpr int UP = 2 * UNROLL;
                const uint16_t* hp[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) hp[mt] = hplane + (size_t)min(mt * kTileM + col, Bg - 1) * ppitch_h;
                const uint16_t* er = reinterpret_cast<const uint16_t*>(erow);
                uint4 eb[UP];
                const int klast = d - VEC;
#pragma unroll
                for (int uu = 0; uu < UP; ++uu) {
                    eb[uu] = *reinterpret_cast<const uint4*>(er + min(uu * KSTEP + kq * VEC, klast));
                    __builtin_amdgcn_sched_barrier(0);
                }
                uint4 hn[MT][3];
                auto read_planes = [&](int k, uint4 (&dst)[MT][3]) {
                    const bool in = k < d;
                    const int kc = in ? k : 0;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int pnum = 0; pnum < 3; ++pnum) {
                            const uint4 h = *reinterpret_cast<const uint4*>(hp[mt] + pnum * plane_stride + kc);
                            dst[mt][pnum] = in ? h : make_uint4(0u, 0u, 0u, 0u);
                        }
                };
                read_planes(kq * VEC, hn);
                for (int ks0 = 0; ks0 < nks; ks0 += UP) {
#pragma unroll
                    for (int uu = 0; uu < UP; ++uu) {
                        const int k = (ks0 + uu) * KSTEP + kq * VEC;
                        uint4 hv[MT][3];
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int pnum = 0; pnum < 3; ++pnum) hv[mt][pnum] = hn[mt][pnum];
                        read_planes(k + KSTEP, hn);
                        const bf16x8 b = __builtin_bit_cast(bf16x8, eb[uu]);
#pragma unroll
                        for (int pnum = 0; pnum < 3; ++pnum)
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    __builtin_bit_cast(bf16x8, hv[mt][pnum]), b, acc[mt], 0, 0, 0);
                        eb[uu] = *reinterpret_cast<const uint4*>(er + min(k + UP * KSTEP, klast));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else if (ALIGNED) {
                // Rolling prefetch: UNROLL candidate-row loads stay in flight all the time.  Slot
                // uu is consumed (LDS read of the hidden rows, VEC matrix instructions) and at
                // once refilled with the chunk UNROLL k-steps ahead, so memory latency and
                // arithmetic overlap inside the wave instead of alternating.  Addresses past
                // the row are clamped into it (no branch around a load); such chunks meet
                // hidden values forced to zero.
                float ev[UNROLL][VEC];
                const int klast = d - VEC;  // d is a multiple of VEC here
#pragma unroll
                for (int uu = 0; uu < UNROLL; ++uu) {
                    ElemTraits<ET>::load16(erow + min(uu * KSTEP + kq * VEC, klast), ev[uu]);
                    __builtin_amdgcn_sched_barrier(0);  // issue order = consumption order
                }
                // the hidden chunk of a slot is read from LDS one slot ahead, so that its latency
                // hides behind the previous slot's matrix instructions
                float hn[MT][VEC];
                auto read_hidden = [&](int k, float (&dst)[MT][VEC]) {
                    const bool in = k < d;
                    const int kc = in ? k : 0;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int q = 0; q < VEC; q += 4) {
                            const float4 h4 = *reinterpret_cast<const float4*>(hrow[mt] + kc + q);
                            dst[mt][q] = in ? h4.x : 0.f; dst[mt][q + 1] = in ? h4.y : 0.f;
                            dst[mt][q + 2] = in ? h4.z : 0.f; dst[mt][q + 3] = in ? h4.w : 0.f;
                        }
                };
                read_hidden(kq * VEC, hn);
                for (int ks0 = 0; ks0 < nks; ks0 += UNROLL) {
#pragma unroll
                    for (int uu = 0; uu < UNROLL; ++uu) {
                        const int k = (ks0 + uu) * KSTEP + kq * VEC;
                        float hv[MT][VEC];
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int q = 0; q < VEC; ++q) hv[mt][q] = hn[mt][q];
                        read_hidden(k + KSTEP, hn);  // next slot (past the row: zeros)
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int q = 0; q < VEC; ++q)
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[mt][q], ev[uu][q], acc[mt], 0, 0, 0);
                        // (unconditional: a branch around the load would make the compiler wait
                        // for every outstanding load at the top of the round; past the end of the
                        // row the clamped address re-reads its last chunk, a cache hit)
                        ElemTraits<ET>::load16(erow + min(k + UNROLL * KSTEP, klast), ev[uu]);
                        // keep the refill here: the scheduler would otherwise sink it towards
                        // its use a round later and leave one or two loads in flight
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
                for (int ks0 = 0; ks0 < nks; ks0 += UNROLL) {
                    float ev[UNROLL][VEC];
#pragma unroll
                    for (int uu = 0; uu < UNROLL; ++uu) {
                        const int k = (ks0 + uu) * KSTEP + kq * VEC;
#pragma unroll
                        for (int q = 0; q < VEC; ++q) ev[uu][q] = (k + q < d) ? elem_f32(erow + k + q) : 0.f;
                    }
#pragma unroll
                    for (int uu = 0; uu < UNROLL; ++uu) {
                        const int k = (ks0 + uu) * KSTEP + kq * VEC;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            float hv[VEC];
#pragma unroll
                            for (int q = 0; q < VEC; ++q)
                                hv[q] = (k + q < d) ? hrow[mt][min(k + q, d - 1)] : 0.f;
#pragma unroll
                            for (int q = 0; q < VEC; ++q)
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[q], ev[uu][q], acc[mt], 0, 0, 0);
                        }
                    }
                }
            }
            LSH_TRACE(1, 3);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = row0 + mt * kTileM + 4 * kq + r, c = n0 + col;
                    const bool valid = row < row0 + Bg && c < C;
                    const float x = acc[mt][r];
                    if (valid) logits[((size_t)s * B + row) * cpitch + c] = x;
                    tile_record_store<false, false>(recs, ((size_t)s * B + row) * recs.pitch + nt, row < row0 + Bg, valid,
                                             x, col, (int32_t)j);
                }
        }
        seg = seg_end;
    }
    LSH_TRACE(1, 4);

    // the remainder: one workgroup per tile, k split over its waves, hidden rows from LDS
    for (uint32_t t = wave_tiles + bx; t < total_tiles; t += (uint32_t)gx) {
        const int s = sentence_of(t);
        stage(s);
        const int nt = (int)(t - tile_pref[s]);
        const int C = count ? count[s] : V;
        const int cidx = min(nt * kTileN + col, C - 1);
        const int64_t j = cand ? cand[(size_t)s * V + cidx] : cidx;
        // (the split-k tile code reads fp32 rows: from global memory when LDS holds bf16 planes)
        logits_tile_all_rows<ET, WAVES, (UNROLL < 4 ? UNROLL : 4), ALIGNED, MT>(
            E, ld, d, H, B, s, nt, C, j, logits, cpitch, recs, red,
            PLANES ? nullptr : hl, PLANES ? 0 : pitch, row0, row0 + Bg);
    }
}

// 33..64 beams, fp32 rows, d <= 1024: the operands change places.  The hidden rows do not fit in
// LDS (64 x 4 KB) and taking them in groups makes every group pull the candidate rows through
// the vector memory path again, which is what bounds that kernel.  Here the HIDDEN rows live in
// registers and the CANDIDATE rows pass through LDS: a workgroup of 16 waves = 4 row groups x 4
// slices of 256 k; wave (g, q) keeps the A operands of rows 16 g .. 16 g + 15, k in [256 q,
// 256 q + 256) in 64 registers for the whole kernel (16 k-steps x 4), and the workgroup walks the
// tiles of its sentence: every wave copies ONE candidate row of the next tile (4 KB, contiguous:
// whole cache lines) into the other half of a double-buffered LDS tile while all waves contract
// the current tile out of LDS (ds_read_b128 = the B operand of four matrix instructions).  A
// candidate row is loaded once per tile, whatever the number of beams.  The partial tiles of
// the four slices are summed through LDS in slice order, the wave of slice q finishing
// accumulator register q of its row group (a quarter of the tile's logits and softmax partials
// each: one wave finishing all of it was the critical path).  One barrier per tile.
// ONE record (max, sum exp) per hidden row for every kGroupTiles tiles the workgroup walks (the
// tiles j0 + (kGroupTiles m + i) G, i < kGroupTiles, at index j0 + m G; select.h): the
// selection's pass over the records is bound by what one CU can pull, and fifty rows of per-tile
// records were 140 KB per sentence.
//   LDS: 2 x 16 rows x 1028 floats (pitch 4 modulo 32: conflict-free 16-byte reads) + 2 x 12 KB of
//   partial tiles = 155.6 KB: one workgroup per CU.  Columns d .. 1023 of the tile are zeroed
//   once (they meet A operands that are zero, and 0 x garbage may be NaN).
//
// UNION: the sentence's candidate list is made here too, from the bitmaps an earlier kernel left
// for the parts of the sentence (k_part_bitmaps) and the top-frequent words: every workgroup ORs
// them in the LDS the tiles will use later, scans the popcounts, and the thread that owns a bit
// whose tile is one of this workgroup's writes its id to the list in memory and, for the
// workgroup's first kEsIdTiles tiles, to a small LDS table (later tiles read their ids back from
// the list).  All this runs while the A operands are on their way; the union kernel, its launch
// and the trip of the list through memory go away.
constexpr int kEsPitch = 1028, kEsSlice = 256, kEsSlices = 4;
constexpr int kEsIdTiles = 16;
constexpr int kEsUnionParts = 6;   // part bitmaps the kernel can OR (64 rows hashed 12 at a time)
// LDS: the two tiles, the partial tiles, the running record of each of the 64 rows (registers are
// all taken), and for UNION the id table.
__host__ __device__ inline size_t estage_lds_bytes(bool with_union = false) {
    return ((size_t)2 * kTileN * kEsPitch + (size_t)2 * 12 * 4 * kWave + 2 * 64 +
            (with_union ? kEsIdTiles * kTileN : 0)) * 4;
}
// LDS words the union needs inside the tile buffers (bitmap + scan scratch)
__host__ __device__ inline size_t estage_union_words(int V) { return (size_t)bitmap_words_padded(V) + 64; }
constexpr int kEsCoopBits = 8;   // list positions of one tile in one thread from which its wave shares the work
struct EstageUnion {
    const uint32_t* parts;    // [S, nparts, ceil(V/32)] bitmaps
    int nparts;
    const int32_t* topfreq;   // [T]
    int T;
    int32_t* cand;            // out: [S, V] ascending candidate ids
    int32_t* count;           // out: [S]
};

template <int MT, bool UNION>
__global__ void __launch_bounds__(1024)
k_logits_estage(const float* __restrict__ E, int64_t ld, int d, const float* __restrict__ H, int S,
                int B, const int32_t* __restrict__ cand, const int32_t* __restrict__ count, int V,
                float* __restrict__ logits, int64_t cpitch, TileRecords recs, EstageUnion un) {
    constexpr int KSTEP = 16, NSTEP = kEsSlice / KSTEP;
    extern __shared__ uint32_t esm[];
    float* etile = reinterpret_cast<float*>(esm);                         // [2][16][kEsPitch]
    float* red = etile + 2 * kTileN * kEsPitch;                           // [2][16 waves][3][64]
    float2* run = reinterpret_cast<float2*>(red + 2 * 12 * 4 * kWave);            // [64 rows] record so far
    uint32_t* ids_lds = reinterpret_cast<uint32_t*>(run + 64);                    // UNION: [kEsIdTiles][16]
    const int tid = threadIdx.x, ln = lane_id(), wv = wave_id();
    const int col = ln & 15, kk = ln >> 4;
    const int g = wv >> 2, q = wv & 3;                                     // row group, k slice
    const int s = blockIdx.x % S, j0 = blockIdx.x / S, G = gridDim.x / S;  // tiles j0, j0 + G, ...

    // A operands: rows 16 g + col (clamped), k = 256 q + 16 step + 4 kk + (0..3); zero past d
    float a[NSTEP][4];
    auto load_a = [&]() {
        const int row = min(g * kTileM + col, B - 1);
        const float* hrow = H + ((size_t)s * B + row) * d;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            const int k = q * kEsSlice + st * KSTEP + 4 * kk;
            const float4 h = *reinterpret_cast<const float4*>(hrow + min(k, d - 4));
            const bool in = k < d && g < MT;
            a[st][0] = in ? h.x : 0.f; a[st][1] = in ? h.y : 0.f;
            a[st][2] = in ? h.z : 0.f; a[st][3] = in ? h.w : 0.f;
        }
    };
    int C;
    if constexpr (UNION) {
        // Loads return in order: everything the union reads is asked for first (the first 4096
        // bitmap words of up to kEsUnionParts parts, the first 3072 top-frequent ids), the A operands
        // after it -- they arrive while the union is being made: the barriers in here are
        // lds_barrier, which does not wait for them.
        uint32_t* bm = esm;
        uint32_t* wsum = bm + bitmap_words_padded(V);
        const int nwords = (V + 31) >> 5;
        const uint32_t* pb = un.parts + (size_t)s * un.nparts * nwords;
        constexpr int SLOTS = 4, PARTS = kEsUnionParts;
        uint32_t pw[SLOTS][PARTS];
#pragma unroll
        for (int u = 0; u < SLOTS; ++u)
#pragma unroll
            for (int b = 0; b < PARTS; ++b) pw[u][b] = 0u;
        // (words past the end repeat the last; parts and slots that do not exist are skipped by
        // uniform branches: a load that hits in cache costs the load path as much as one that misses)
#pragma unroll
        for (int u = 0; u < SLOTS; ++u) {
            if (u * 1024 >= nwords) break;
#pragma unroll
            for (int b = 0; b < PARTS; ++b) {
                if (b >= un.nparts) break;
                pw[u][b] = pb[(size_t)b * nwords + min(tid + u * 1024, nwords - 1)];
            }
        }
        const int32_t tf0 = (tid < un.T) ? un.topfreq[tid] : -1;
        const int32_t tf1 = (tid + 1024 < un.T) ? un.topfreq[tid + 1024] : -1;
        const int32_t tf2 = (tid + 2048 < un.T) ? un.topfreq[tid + 2048] : -1;
        __builtin_amdgcn_sched_barrier(0);   // (issue order = the order written here)
        load_a();
#pragma unroll
        for (int u = 0; u < SLOTS; ++u) {
            uint32_t x = 0;
#pragma unroll
            for (int b = 0; b < PARTS; ++b) x |= pw[u][b];
            if (tid + u * 1024 < nwords) bm[tid + u * 1024] = x;
        }
        for (int i = tid + SLOTS * 1024; i < nwords; i += 1024) {
            uint32_t x = 0;
            for (int b = 0; b < un.nparts; ++b) x |= pb[(size_t)b * nwords + i];   // (nparts <= kEsUnionParts)
            bm[i] = x;
        }
        lds_barrier();
        LSH_TRACE(1, 13);
        if (un.T > 0) mark_ids_of_wave(bm, V, tf0);
        if (un.T > 1024) mark_ids_of_wave(bm, V, tf1);
        if (un.T > 2048) mark_ids_of_wave(bm, V, tf2);
        for (int i = 3072 + tid; i - tid < un.T; i += 1024) mark_ids_of_wave(bm, V, (i < un.T) ? un.topfreq[i] : -1);
        lds_barrier();
        const int per_thread = (nwords + 1023) / 1024;
        const int wbeg = min(tid * per_thread, nwords), wend = min(wbeg + per_thread, nwords);
        uint32_t mine = 0;
        for (int i = wbeg; i < wend; ++i) mine += __popc(bm[i]);
        uint32_t total;
        uint32_t pos = block_incl_scan<true>(mine, wsum, &total) - mine;   // list position of my first bit
        C = (int)total;
        LSH_TRACE(1, 14);
        // my bits are list positions [pos, pos + mine); of the tiles they fall into, this
        // workgroup's are those congruent to j0 modulo G.  A thread with a few positions of such a
        // tile skips to its first bit (whole words by popcount) and writes the ids out itself; one
        // with kEsCoopBits or more (the dense words of the top-frequent ids put a whole tile into
        // one thread) hands them to the lanes of its wave, each finding one id by rank -- sixteen
        // dependent steps of a single lane, in every workgroup, used to be most of this phase.
        {
            const uint32_t end = pos + mine;
            const int t0 = (int)(pos >> 4);
            int nt = t0 + (j0 - t0 % G + G) % G;
            int k = nt / G;
            auto pending = [&]() { return mine != 0u && (uint32_t)nt * kTileN < end; };
            while (__ballot(pending()) != 0ull) {   // (uniform)
                const bool has = pending();
                const uint32_t lo = has ? max(pos, (uint32_t)nt * kTileN) : 0u;
                const uint32_t hi = has ? min(end, (uint32_t)nt * kTileN + kTileN) : 0u;
                const uint32_t n = hi - lo;
                if (has && n < (uint32_t)kEsCoopBits) {
                    uint32_t skip = lo - pos;
                    int i = wbeg;
                    uint32_t bits = bm[i];
                    for (uint32_t c = __popc(bits); skip >= c; c = __popc(bits)) { skip -= c; bits = bm[++i]; }
                    for (; skip; --skip) bits &= bits - 1u;
                    for (uint32_t at = lo; at < hi; ++at) {
                        while (!bits) bits = bm[++i];
                        const int32_t id = (i << 5) + (__ffs(bits) - 1);
                        bits &= bits - 1u;
                        un.cand[(size_t)s * V + at] = id;
                        if (k < kEsIdTiles) ids_lds[k * kTileN + (int)(at & 15u)] = (uint32_t)id;
                    }
                }
                for (uint64_t heavy = __ballot(has && n >= (uint32_t)kEsCoopBits); heavy; heavy &= heavy - 1) {   // (uniform)
                    const int o = __ffsll((unsigned long long)heavy) - 1;
                    const uint32_t o_lo = wave_read_lane(lo, o), o_n = wave_read_lane(n, o), o_pos = wave_read_lane(pos, o);
                    const int o_k = (int)wave_read_lane((uint32_t)k, o);
                    int i = (int)wave_read_lane((uint32_t)wbeg, o);
                    if ((uint32_t)ln < o_n) {
                        uint32_t r = o_lo - o_pos + (uint32_t)ln;      // my bit's rank in the owner's words
                        uint32_t bits = bm[i];
                        for (uint32_t c = __popc(bits); r >= c; c = __popc(bits)) { r -= c; bits = bm[++i]; }
                        const int32_t id = (i << 5) + (int32_t)nth_set_bit(bits, r);
                        const uint32_t at = o_lo + (uint32_t)ln;
                        un.cand[(size_t)s * V + at] = id;
                        if (o_k < kEsIdTiles) ids_lds[o_k * kTileN + (int)(at & 15u)] = (uint32_t)id;
                    }
                }
                if (has) { nt += G; ++k; }
            }
        }
        LSH_TRACE(1, 15);
        if (j0 == 0 && tid == 0) un.count[s] = C;
        lds_barrier();   // the table is written and the bitmap done with (the ids of later tiles are read
                         // back from the list only after many full barriers)
    } else {
        C = count ? count[s] : V;
    }
    const int ntiles = (C + kTileN - 1) / kTileN;
    if (j0 >= ntiles) return;                                             // (whole workgroup)
    LSH_TRACE(1, 0);

    // this wave's candidate row of a tile, 4 KB as up to four 16-byte loads per lane
    const int d4 = d >> 2;
    auto id_of = [&](int nt) -> int64_t {                                  // (any nt >= 0)
        if constexpr (UNION) {
            // (waves past the end of the list, and tiles past the last, take a candidate that
            // exists: their rows are never stored)
            if (nt >= ntiles) nt = j0;
            const int cidx = nt * kTileN + (nt * kTileN + wv < C ? wv : 0);
            const int k = (nt - j0) / G;
            return k < kEsIdTiles ? (int64_t)ids_lds[k * kTileN + (cidx & 15)] : (int64_t)un.cand[(size_t)s * V + cidx];
        }
        const int cidx = min(nt * kTileN + wv, C - 1);                     // clamped rows are never stored
        return cand ? (int64_t)cand[(size_t)s * V + cidx] : (int64_t)cidx;
    };
    auto row_of = [&](int64_t j) { return reinterpret_cast<const float4*>(E + j * ld); };
    float4 st0, st1, st2, st3;   // (named registers: an array captured by the lambdas goes to scratch)
    const int c0 = min(ln, d4 - 1), c1 = min(ln + kWave, d4 - 1), c2 = min(ln + 2 * kWave, d4 - 1),
              c3 = min(ln + 3 * kWave, d4 - 1);
    auto load_row = [&](const float4* r) { st0 = r[c0]; st1 = r[c1]; st2 = r[c2]; st3 = r[c3]; };
    auto store_row = [&](int buf) {
        float4* dst = reinterpret_cast<float4*>(etile + ((size_t)buf * kTileN + wv) * kEsPitch);
        if (ln < d4) dst[ln] = st0;
        if (ln + kWave < d4) dst[ln + kWave] = st1;
        if (ln + 2 * kWave < d4) dst[ln + 2 * kWave] = st2;
        if (ln + 3 * kWave < d4) dst[ln + 3 * kWave] = st3;
    };
    load_row(row_of(id_of(j0)));
    int64_t id_next = id_of(j0 + G);   // candidate ids are fetched a tile ahead of their rows
    if constexpr (!UNION) load_a();
    // zero the columns d .. 1023 of both buffers (never written by the row copies)
    {
        const int padw = kEsSlices * kEsSlice - d;                         // a multiple of 4, < 1024
        for (int e = tid; e < 2 * kTileN * padw; e += 1024) {
            const int r = e / padw, c = e - r * padw;
            etile[(size_t)r * kEsPitch + d + c] = 0.f;
        }
    }
    LSH_TRACE(1, 1);
    store_row(0);
    __syncthreads();
    LSH_TRACE(1, 2);

    int buf = 0;
    // (max, sum exp) of a row over the tiles of the current group: kept in LDS by the lane that
    // writes the row's records (column 0), which alone reads and writes its slot
    if (g < MT && col == 0) run[g * kTileM + 4 * kk + q] = make_float2(-INFINITY, 0.f);
    int kt = 0;                                 // tiles done
    for (int nt = j0; nt < ntiles; nt += G, buf ^= 1, ++kt) {
        const bool more = nt + G < ntiles;
        if (more) {                                                        // in flight during the contraction
            load_row(row_of(id_next));
            id_next = id_of(nt + 2 * G);
        }
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        if (g < MT) {
            const float* bt = etile + ((size_t)buf * kTileN + col) * kEsPitch + q * kEsSlice + 4 * kk;
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                const float4 b = *reinterpret_cast<const float4*>(bt + st * KSTEP);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[st][0], b.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[st][1], b.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[st][2], b.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[st][3], b.w, acc, 0, 0, 0);
            }
            // the wave of slice q finishes accumulator register q of its row group (rows 16 g +
            // 4 kk + q): it keeps that register and leaves the other three for its siblings
            float* rp = red + (((size_t)buf * 16 + wv) * 3) * kWave;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (r != q) rp[(r < q ? r : r - 1) * kWave + ln] = acc[r];
        }
#ifdef LSHBEAM_TRACE
        if ((nt - j0) / G < 5) LSH_TRACE(1, 3 + 2 * ((nt - j0) / G));
#endif
        if (more) store_row(buf ^ 1);   // the other half was last read before the previous barrier
        __syncthreads();
#ifdef LSHBEAM_TRACE
        if ((nt - j0) / G < 5) LSH_TRACE(1, 4 + 2 * ((nt - j0) / G));
#endif
        if (g < MT) {
            // x = sum over the four slices in slice order (this wave's own share in its place)
            const float own = (q == 0) ? acc[0] : (q == 1) ? acc[1] : (q == 2) ? acc[2] : acc[3];
            float x = 0.f;
#pragma unroll
            for (int qq = 0; qq < kEsSlices; ++qq) {
                float part = own;
                if (qq != q)   // wave-uniform
                    part = red[(((size_t)buf * 16 + (g * 4 + qq)) * 3 + (q < qq ? q : q - 1)) * kWave + ln];
                x = (qq == 0) ? part : x + part;
            }
            const int n0 = nt * kTileN;
            const int row = g * kTileM + 4 * kk + q, c = n0 + col;
            const bool valid = row < B && c < C;
            if (valid) logits[((size_t)s * B + row) * cpitch + c] = x;
            const float mx = row16_max(valid ? x : -INFINITY);
            const float se = row16_sum(valid ? expf(x - mx) : 0.f);
            if (col == 0) {
                // (one fast exponential, no branch: 16 waves share the CU's issue slots, and every
                // instruction here is paid once per tile by each of them)
                float2 acc2 = run[g * kTileM + 4 * kk + q];
                const float hi = fmaxf(acc2.x, mx);
                const float e = __expf(fminf(acc2.x, mx) - hi);      // exp(-|difference|); 0 for the first tile
                acc2.y = (mx > acc2.x) ? fmaf(acc2.y, e, se) : fmaf(se, e, acc2.y);
                acc2.x = hi;
                const bool group_end = kt % kGroupTiles == kGroupTiles - 1 || !more;
                if (group_end && row < B)
                    reinterpret_cast<float2*>(recs.rec)[((size_t)s * B + row) * recs.pitch + j0 +
                                                        (size_t)(kt / kGroupTiles) * G] = acc2;
                run[g * kTileM + 4 * kk + q] = group_end ? make_float2(-INFINITY, 0.f) : acc2;
            }
        }
    }
}

}  // namespace lshbeam
