// Host-only check of the index arithmetic the kernels share with the host: workspace carving and
// the LDS plans of every kernel, over the extreme shapes the library accepts (B = 256, S = 4096,
// V = 2^24, d not a multiple of 4).  Built by tests/test_host_plans.py with hipcc
// and run on the CPU; no GPU call is made (the kernels in the headers are compiled but never launched).  Every region must start aligned, lie behind its
// predecessor and end inside what the size function reports.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_1806_00588_amd/csrc/candidates.h"
#include "../paper_1806_00588_amd/csrc/fused.h"
#include "../paper_1806_00588_amd/csrc/logits.h"
#include "../paper_1806_00588_amd/csrc/select.h"
#include "../paper_1806_00588_amd/csrc/workspace.h"

using namespace lshbeam;

static int failures = 0;
#define CHECK(cond, ...)                                                  \
    do {                                                                  \
        if (!(cond)) {                                                    \
            ++failures;                                                   \
            std::printf("FAILED %s:%d  %s  ", __FILE__, __LINE__, #cond); \
            std::printf(__VA_ARGS__);                                     \
            std::printf("\n");                                            \
        }                                                                 \
    } while (0)

constexpr size_t kLdsLimit = 160 * 1024 - 1024;   // what the host allows a kernel to ask for

static void check_workspace(int S, int B, int V, bool full) {
    char* base = reinterpret_cast<char*>((uintptr_t)1 << 40);   // never dereferenced
    const Workspace w = carve_workspace(S, B, V, full, base);
    const size_t R = (size_t)S * B;
    struct Region { const char* name; const void* p; size_t bytes; };
    const Region regs[] = {
        {"cand", w.cand, full ? 0 : (size_t)S * V * 4},
        {"count", w.count, (size_t)S * 4},
        {"logits", w.logits, R * (size_t)w.cpitch * 4},
        {"partials", w.partials, R * (size_t)w.ppitch * sizeof(TileRecord)},
        {"ids2", w.ids2, R * (size_t)w.ppitch * 4},
        {"lse", w.lse, R * 4},
        {"row_bitmaps", w.row_bitmaps, full ? 0 : R * (((size_t)V + 31) / 32) * 4},
    };
    const char* prev_end = base;
    for (const Region& r : regs) {
        const char* p = (const char*)r.p;
        CHECK(((uintptr_t)p % kAlign) == 0, "%s misaligned (S=%d B=%d V=%d)", r.name, S, B, V);
        CHECK(p >= prev_end, "%s overlaps its predecessor (S=%d B=%d V=%d)", r.name, S, B, V);
        CHECK(p + r.bytes <= base + w.bytes, "%s ends outside the workspace (S=%d B=%d V=%d)", r.name, S, B, V);
        CHECK(r.bytes / 4 <= w.bytes, "size overflow in %s", r.name);
        prev_end = p + r.bytes;
    }
    CHECK(w.cpitch >= V && w.cpitch % 64 == 0 && w.ppitch * kTileN >= w.cpitch && w.ppitch >= kMaxFusedGrid,
          "pitches V=%d", V);
    // forced narrow tiles of the fused plans: never more tiles than records fit in a row
    for (int C : {0, 1, 5, 100, 2224, 4095, 4096, V / 2, V})
        for (int forced : {0, 1, 3, 9, 16, 40}) {
            if (C > V) continue;
            const int tn = select_tile_width(C, forced, w.ppitch);
            CHECK(tn >= 1 && tn <= 16, "tile width %d", tn);
            CHECK(((int64_t)C + tn - 1) / tn <= w.ppitch, "tiles beyond the record pitch (C=%d forced=%d V=%d)", C, forced, V);
        }
    // the largest index any kernel forms: row R-1, last column / last tile
    CHECK((R - 1) * (size_t)w.cpitch + (size_t)V - 1 < R * (size_t)w.cpitch, "logit index");
    CHECK((size_t)(((size_t)V + 15) / 16) <= (size_t)w.ppitch, "tile count exceeds the record pitch V=%d", V);
}

// the LDS regions of build_presence_bitmap / k_candidates / k_cand_logits, as the kernels lay them out
static void check_candidate_lds(int V, int d, int P, int K, int W, int B) {
    const int mn = candidates_min_stage(d);
    CHECK(mn >= d && mn % 4 == 0, "min stage d=%d", d);
    for (int stage : {mn, mn + 4 * 1000, (int)((kLdsLimit / 4 - (bitmap_words_padded(V) + (size_t)P * K + 3 * kCandThreads + 64)) & ~(size_t)3)}) {
        if (stage < mn) continue;
        const size_t total = candidates_lds_words(V, P, K, stage);
        if (total * 4 > kLdsLimit) continue;   // the host refuses such a plan
        const size_t bmw = bitmap_words_padded(V);
        CHECK(bmw * 32 >= (size_t)V && bmw % 4 == 0, "bitmap words V=%d", V);
        const size_t stage_at = bmw, perms_at = stage_at + stage, start_at = perms_at + (size_t)P * K;
        const size_t band_at = start_at + kCandThreads, pref_at = band_at + kCandThreads, wsum_at = pref_at + kCandThreads;
        CHECK(wsum_at + 64 == total, "candidate regions do not add up (V=%d P=%d K=%d)", V, P, K);
        CHECK(stage_at % 4 == 0, "stage not 16-byte aligned");
        const int rows = candidates_rows_per_chunk(B, d, W, stage);
        CHECK(rows >= 1 && rows <= B, "rows per chunk %d (B=%d)", rows, B);
        CHECK((size_t)rows * d <= (size_t)stage, "chunk of %d rows x %d does not fit a stage of %d", rows, d, stage);
        CHECK(rows * W <= kCandThreads, "pairs of a chunk exceed the workgroup (rows=%d W=%d)", rows, W);
        CHECK(rows * P <= kCandThreads || true, "-");
        // fused kernel: prefix array and reduction buffer behind the candidate regions; the
        // selection's shared state from the start
        const size_t fused = fused_lds_words(V, P, K, stage);
        CHECK(total + kFusedTileIdWords + (size_t)kFusedWaves * 4 * kWave <= fused, "fused regions (V=%d)", V);
        CHECK(total % 4 == 0 || true, "-");
        CHECK(fused >= kSelSharedWords, "fused LDS smaller than the selection's state");
        // k_candidates reuses the stage for the dense-word list: stage / 2 entries of 8 bytes
        CHECK((size_t)(stage / 2) * 2 <= (size_t)stage, "dense list");
    }
    const size_t un = union_logits_lds_words(V);
    CHECK(bitmap_words_padded(V) + 64 + kFusedTileIdWords + (size_t)kFusedWaves * 4 * kWave <= un, "union regions V=%d", V);
    CHECK(un >= kSelSharedWords, "union LDS smaller than the selection's state");
    CHECK(union_compact_lds_words(V) == (size_t)bitmap_words_padded(V) + 64 + 2 * (size_t)kUnionDenseCap, "union compact V=%d", V);
}

static void check_hit_rows(int V, int d, int P) {
    const int vq = hit_slice_words(V);
    CHECK(vq % 128 == 0 && (size_t)vq * kHitSlices >= (size_t)V, "slices do not cover V=%d", V);
    CHECK((size_t)vq * (kHitSlices - 1) < (size_t)V + 128 * kHitSlices, "slices far beyond V=%d", V);
    const size_t fixed = hit_rows_fixed_lds_words(V, d, P);
    const size_t counters = (size_t)vq / 2, row = (size_t)((d + 3) & ~3), codes = ((size_t)P + 1) / 2;
    CHECK(counters + row + codes + 32 + (kCandThreads + 64) + 2 * (size_t)kCandThreads <= fixed,
          "hit-row regions exceed their size (V=%d d=%d P=%d)", V, d, P);
}

static void check_hlds(int S, int rows, int d) {
    for (int waves : {8, 16})
        for (bool planes : {false, true}) {
            const size_t bytes = hlds_lds_bytes(S, rows, d, waves, planes);
            const size_t pref = (size_t)((S + 1 + 3) & ~3), red = (size_t)waves * 4 * kWave;
            const size_t hidden = planes ? (size_t)rows * hlds_pitch_planes(d) * 6 : (size_t)rows * hlds_pitch(d) * 4;
            CHECK((pref + red) * 4 + hidden == bytes, "hlds regions (S=%d rows=%d d=%d)", S, rows, d);
            CHECK(hlds_pitch(d) >= d && hlds_pitch(d) % 32 == 4, "hlds pitch d=%d", d);
            CHECK(hlds_pitch_planes(d) >= d && hlds_pitch_planes(d) % 64 == 8, "plane pitch d=%d", d);
            CHECK(((pref + red) * 4) % 16 == 0, "hidden rows not 16-byte aligned in LDS");
        }
}

// small_div() of the kernels: (int)((x + 0.5f) * r) with r = the hardware's reciprocal of y, which may
// differ from the correctly rounded 1 / y by one unit in the last place; checked here with r two
// units off either way, for every x < 1024 and y <= 1024.
static void check_small_div_margin() {
    for (int y = 1; y <= 1024; ++y) {
        const float exact = 1.0f / (float)y;
        float lo = exact, hi = exact;
        for (int i = 0; i < 2; ++i) { lo = std::nextafterf(lo, 0.0f); hi = std::nextafterf(hi, 2.0f); }
        for (float r : {lo, exact, hi})
            for (int x = 0; x < 1024; ++x)
                CHECK((int)(((float)x + 0.5f) * r) == x / y, "small_div x=%d y=%d", x, y);
    }
}

// nth_set_bit() against a bit-by-bit walk: every rank of a few thousand words (all one-bit and
// two-bit words, dense and random ones).
static void check_nth_set_bit() {
    std::vector<uint32_t> words = {0xFFFFFFFFu, 0x80000000u, 0x00000001u, 0xAAAAAAAAu, 0x55555555u, 0xFFFF0000u, 0x0000FFFFu};
    for (int a = 0; a < 32; ++a)
        for (int b = a; b < 32; ++b) words.push_back((1u << a) | (1u << b));
    uint64_t x = 0x9E3779B97F4A7C15ull;
    for (int i = 0; i < 4000; ++i) { x ^= x << 13; x ^= x >> 7; x ^= x << 17; words.push_back((uint32_t)(x >> 16)); }
    for (uint32_t w : words) {
        uint32_t r = 0;
        for (uint32_t bit = 0; bit < 32; ++bit)
            if (w >> bit & 1u) { CHECK(nth_set_bit(w, r) == bit, "nth_set_bit(%08x, %u)", w, r); ++r; }
    }
}

int main() {
    check_small_div_margin();
    check_nth_set_bit();
    // workspace: the largest accepted S, B, V and their neighbours, ragged V
    for (int V : {1, 15, 16, 17, 63, 64, 65, 1000, 40000, 100000, 200000, (1 << 24) - 1, 1 << 24})
        for (int S : {1, 2, 64, 4096})
            for (int B : {1, 12, 17, 50, 256})
                for (bool full : {false, true}) {
                    if ((size_t)S * B * V > ((size_t)1 << 45)) continue;   // (keeps sizes below 2^48 bytes)
                    check_workspace(S, B, V, full);
                }
    check_workspace(4096, 256, 1 << 20, false);
    check_workspace(1, 256, 1 << 24, false);
    check_workspace(4096, 1, 1 << 24, true);
    // LDS plans: vocabulary sizes up to what fits a bitmap in LDS, odd hidden sizes, many codes
    for (int V : {1, 31, 32, 33, 1000, 40000, 100000, 200000, 1000000})
        for (int d : {8, 50, 64, 77, 1000, 1024, 1026, 4099, 20000})
            for (int W : {1, 4, 8, 16, 500, 1024})
                for (int K : {2, 8, 16}) {
                    if (K > d) continue;
                    const int P = W * 3;
                    for (int B : {1, 12, 29, 32, 50, 256}) check_candidate_lds(V, d, P, K, W, B);
                    check_hit_rows(V, d, P);
                }
    for (int S : {1, 32, 64, 4096})
        for (int rows : {1, 10, 16, 32})
            for (int d : {8, 50, 1000, 1024, 1026, 4099}) check_hlds(S, rows, d);
    CHECK(estage_lds_bytes() <= kLdsLimit, "estage LDS");
    CHECK(sizeof(SelShared) + 1024 <= 64 * 1024, "static LDS of the selection kernel");
    CHECK(kSelSharedWords * 4 >= sizeof(SelShared), "selection state words");
    if (failures) {
        std::printf("%d check(s) failed\n", failures);
        return 1;
    }
    std::printf("host plans ok\n");
    return 0;
}
