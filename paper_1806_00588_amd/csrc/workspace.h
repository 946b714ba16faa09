// Layout of a decode step's workspace (host side): which kernel output lives where in the
// caller's buffer.  Sized for the worst case, a candidate list of all V words, so that a step
// never allocates.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "logits.h"
#include "select.h"

namespace lshbeam {

constexpr size_t kAlign = 256;   // every region starts on a multiple of this (and so must the buffer)
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Workspace {
    int32_t* cand;       // [S, V]
    int32_t* count;      // [S]
    float* logits;       // [R, cpitch]
    TileRecord* partials;  // [R, ppitch]  per (row, tile): fused kernels a TileRecord, the others a float2
                           //   (max, sum exp(logit - max)) in the same place
    int32_t* ids2;       // [R, ppitch]  fused kernels: word id of each record's second largest
    uint32_t* row_bitmaps;  // [R, ceil(V/32)]  per-row (t > 1) or per-part (many beams) bitmaps
    float* lse;          // [R]
    int64_t ppitch;      // tile records per row: cpitch / 16, at least kMaxFusedGrid (narrow tiles)
    int64_t cpitch;      // logits per row: V rounded up to 64
    size_t bytes;
    TileRecords records() const { return TileRecords{partials, ids2, ppitch}; }
};

// S sentences of B beams over a vocabulary of V words; base may be null (sizes only).
inline Workspace carve_workspace(int S_, int B_, int V_, bool full_vocab, void* base) {
    Workspace w{};
    const size_t S = (size_t)S_, B = (size_t)B_, R = S * B, V = (size_t)V_;
    w.cpitch = (int64_t)((V + 63) / 64 * 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return (char*)base + o; };
    w.cand = (int32_t*)take(full_vocab ? 0 : S * V * sizeof(int32_t));
    w.count = (int32_t*)take(S * sizeof(int32_t));
    w.ppitch = w.cpitch / kTileN > kMaxFusedGrid ? w.cpitch / kTileN : (int64_t)kMaxFusedGrid;
    w.logits = (float*)take(R * (size_t)w.cpitch * sizeof(float));
    w.partials = (TileRecord*)take(R * (size_t)w.ppitch * sizeof(TileRecord));
    w.ids2 = (int32_t*)take(R * (size_t)w.ppitch * sizeof(int32_t));
    w.lse = (float*)take(R * sizeof(float));
    w.row_bitmaps = (uint32_t*)take(full_vocab ? 0 : R * ((V + 31) / 32) * sizeof(uint32_t));
    w.bytes = off;
    return w;
}

}  // namespace lshbeam
