// Device-side construction of the per-band bucket tables and cuckoo tables (section "Cuckoo
// lookup", first step: T_w = {band code: [word ids]} flattened, CuckooT_w = {band code:
// (start, length)}).
//
//   1. One 64-bit key per (band, word): band | band code | word id, most significant first.
//      A single radix sort of all W*V keys groups every band's words by code with ids ascending
//      inside a code (the sort is a library primitive, hipCUB; only the bits in use are sorted).
//   2. Position p of the sorted array belongs to band p / V: the id field is the band's flat
//      word array; a position whose code differs from its predecessor's starts a span.
//   3. An exclusive scan of the span-start flags numbers the spans ("keys") of all bands; each
//      start writes (code, start) of its key, the length is the distance to the next start.
//   4. Cuckoo insertion, one thread per key, all bands at once (Alcantara et al.'s scheme for
//      two hash functions): a thread swaps its item into its first slot with a 64-bit
//      atomicExch; if that evicts an item, the thread carries the evicted item to that item's
//      other slot, and so on.  A chain longer than the limit marks the band as failed; the host
//      draws new hash parameters for failed bands and only those are redone.
//   5. The 8-byte (code, key index) words are expanded into the 16-byte slots the probe reads.
#pragma once
#include "candidates.h"

namespace lshbeam {

constexpr uint64_t kCuckooEmpty = ~0ull;

struct SortKeyLayout {
    int id_bits, code_bits;  // key = band << (id_bits + code_bits) | code << id_bits | id
};

__global__ void __launch_bounds__(256)
k_make_sort_keys(const int32_t* __restrict__ codes /*[V, W]*/, int64_t V, int W, SortKeyLayout lay,
                 uint64_t* __restrict__ keys /*[W * V]*/) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // = j * W + w
    if (idx >= V * W) return;
    const int64_t j = idx / W;
    const int w = (int)(idx - j * W);
    const uint64_t code = (uint64_t)(uint32_t)codes[idx];
    keys[(int64_t)w * V + j] =
        ((uint64_t)w << (lay.id_bits + lay.code_bits)) | (code << lay.id_bits) | (uint64_t)j;
}

// words[p] = id field; head[p] = 1 iff p starts a span (first of its band, or a new code).
__global__ void __launch_bounds__(256)
k_split_sorted(const uint64_t* __restrict__ sorted, int64_t V, int W, SortKeyLayout lay,
               int32_t* __restrict__ words, uint32_t* __restrict__ head) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= V * W) return;
    const uint64_t k = sorted[p];
    words[p] = (int32_t)(k & ((1ull << lay.id_bits) - 1ull));
    // band and code together: everything above the id field
    head[p] = (p % V == 0 || (k >> lay.id_bits) != (sorted[p - 1] >> lay.id_bits)) ? 1u : 0u;
}

// Every span start writes its key: code, start inside the band, band.
__global__ void __launch_bounds__(256)
k_emit_keys(const uint64_t* __restrict__ sorted, const uint32_t* __restrict__ head,
            const uint32_t* __restrict__ key_index /*exclusive scan of head*/, int64_t V, int W,
            SortKeyLayout lay, int32_t* __restrict__ key_code, uint32_t* __restrict__ key_start,
            int32_t* __restrict__ key_band) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= V * W || !head[p]) return;
    const uint32_t k = key_index[p];
    const int w = (int)(p / V);
    key_code[k] = (int32_t)((sorted[p] >> lay.id_bits) & ((1ull << lay.code_bits) - 1ull));
    key_start[k] = (uint32_t)(p - (int64_t)w * V);
    key_band[k] = w;
}

// Length of key k's span: up to the next key of the same band, or to the end of the band.
__global__ void __launch_bounds__(256)
k_key_lengths(const uint32_t* __restrict__ key_start, const int32_t* __restrict__ key_band,
              uint32_t n_keys, uint32_t V, uint32_t* __restrict__ key_len) {
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_keys) return;
    const bool last = (k + 1 == n_keys) || key_band[k + 1] != key_band[k];
    key_len[k] = (last ? V : key_start[k + 1]) - key_start[k];
}

// table[i] = empty for the slots of the bands flagged in `redo` (all bands if redo == nullptr).
__global__ void __launch_bounds__(256)
k_cuckoo_clear(uint64_t* __restrict__ table, const BandMeta* __restrict__ bands,
               const uint32_t* __restrict__ band_cap, int W, const uint32_t* __restrict__ redo) {
    const int w = blockIdx.y;
    if (w >= W || (redo && !redo[w])) return;
    const uint32_t cap = band_cap[w];
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < cap; i += gridDim.x * blockDim.x)
        table[bands[w].slot_off + i] = kCuckooEmpty;
}

// One thread per key.  Item = code << 32 | key index.  `failed[w]` is set when a chain in band w
// exceeds max_chain (the item in hand is dropped: the band is redone with new parameters).
__global__ void __launch_bounds__(256)
k_cuckoo_insert(uint64_t* __restrict__ table, const BandMeta* __restrict__ bands,
                const int32_t* __restrict__ key_code, const int32_t* __restrict__ key_band,
                uint32_t n_keys, int max_chain, const uint32_t* __restrict__ redo,
                uint32_t* __restrict__ failed) {
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_keys) return;
    const int w = key_band[k];
    if (redo && !redo[w]) return;
    const BandMeta m = bands[w];
    uint64_t item = ((uint64_t)(uint32_t)key_code[k] << 32) | (uint64_t)k;
    uint32_t pos = cuckoo_hash(m.a0, m.b0, (uint32_t)key_code[k], m.shift);
    for (int step = 0; step < max_chain; ++step) {
        const uint64_t old = atomicExch((unsigned long long*)&table[m.slot_off + pos],
                                        (unsigned long long)item);
        if (old == kCuckooEmpty) return;
        item = old;  // carry the evicted item to its other slot
        const uint32_t code = (uint32_t)(old >> 32);
        const uint32_t h0 = cuckoo_hash(m.a0, m.b0, code, m.shift);
        const uint32_t h1 = cuckoo_hash(m.a1, m.b1, code, m.shift);
        pos = (pos == h0) ? h1 : h0;
    }
    failed[w] = 1u;
}

// Where the vocabulary slices 1, 2, 3 of the hit-count kernel begin inside key k's span (ids are
// ascending inside a span): lower bounds of slice * slice_ids, relative to the span's start.
__global__ void __launch_bounds__(256)
k_slice_cuts(const int32_t* __restrict__ words, const uint32_t* __restrict__ key_start,
             const uint32_t* __restrict__ key_len, const int32_t* __restrict__ key_band,
             uint32_t n_keys, uint32_t V, int slice_ids, uint4* __restrict__ key_cut) {
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_keys) return;
    const int32_t* span = words + (size_t)key_band[k] * V + key_start[k];
    const uint32_t len = key_len[k];
    uint32_t cut[3];
    for (int q = 1; q <= 3; ++q) {
        const int32_t bound = q * slice_ids;
        uint32_t lo = 0, hi = len;  // first position whose id is >= bound
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (span[mid] < bound) lo = mid + 1; else hi = mid;
        }
        cut[q - 1] = lo;
    }
    key_cut[k] = make_uint4(cut[0], cut[1], cut[2], len);
}

// 8-byte table words -> the 16-byte slots of the probe (and the slice cuts beside them).
__global__ void __launch_bounds__(256)
k_cuckoo_finalize(const uint64_t* __restrict__ table, uint64_t n_slots,
                  const uint32_t* __restrict__ key_start, const uint32_t* __restrict__ key_len,
                  const uint4* __restrict__ key_cut, Slot* __restrict__ slots,
                  uint4* __restrict__ cuts) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_slots) return;
    const uint64_t e = table[i];
    Slot s{-1, 0u, 0u, 0u};
    uint4 c = make_uint4(0u, 0u, 0u, 0u);
    if (e != kCuckooEmpty) {
        const uint32_t k = (uint32_t)e;
        s.key = (int32_t)(uint32_t)(e >> 32);
        s.start = key_start[k];
        s.len = key_len[k];
        c = key_cut[k];
    }
    slots[i] = s;
    cuts[i] = c;
}

}  // namespace lshbeam
