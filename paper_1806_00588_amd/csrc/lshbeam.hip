// C ABI of the lshbeam library (see include/lshbeam.h): table build, decode step, beam
// bookkeeping, inspection.  gfx950 only.  Host side: argument validation, the choice of the
// launch plan, kernel launches, the hash parameters of the cuckoo tables (and a host fallback of
// the table build).  Every per-step computation runs in the HIP kernels of candidates.h /
// fused.h / logits.h / select.h / beam.h, the table build in those of build_tables.h.
#include "../../include/lshbeam.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <cctype>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include <hipcub/hipcub.hpp>

#include "beam.h"
#include "build_tables.h"
#include "candidates.h"
#include "fused.h"
#include "logits.h"
#include "select.h"
#include "workspace.h"

using namespace lshbeam;

// Working memory of lsh_decode_step_static, the variant of the decode step for callers that
// cannot allocate: one array per GPU, part of the loaded code object, held until the process
// ends.  In host code `scratch` only names the symbol; the memory of the current device's copy is
// found once per device by scratch_of_device() and kernels are handed that address.
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];   // device address of `scratch` on each GPU, or null

// Address of the current device's copy of `scratch` (the device must be current: each GPU holds
// its own copy at its own address).
hipError_t scratch_of_device(int dev, void** out) {
    *out = nullptr;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_addr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

constexpr int kMaxV = 1 << 24;
constexpr int kMaxB = 256;
constexpr size_t kMaxDynLds = 160 * 1024 - 1024;
constexpr int kTicketSlots = 256;   // workspaces per handle that can take the one-launch plan
constexpr int kTicketBlock = 64;    // counters per workspace = sentences of a fused step at most


struct HostBand {
    std::vector<int32_t> keys;     // distinct band codes, ascending
    std::vector<int32_t> offsets;  // keys.size() + 1 span boundaries into the band's word array
    int capacity = 0;
    BandMeta meta{};
};

// Launch-plan options of a handle (lsh_set_option); kAuto = the library's own rule.
enum Opt {
    kOptFused, kOptFusedGrid, kOptLogitsGrid, kOptLogitsWaves, kOptLogitsHlds, kOptLogitsEstage,
    kOptHldsRem, kOptLogitsPlanes, kOptHldsRows, kOptPartRows, kOptStageRows, kOptOneLaunch, kOptFusedTile,
    kOptEstageUnion, kNumOpts
};
constexpr int kAuto = -1;
const char* const kOptNames[kNumOpts] = {
    "fused", "fused_grid", "logits_grid", "logits_waves", "logits_hlds", "logits_estage",
    "hlds_rem", "logits_planes", "hlds_rows", "part_rows", "stage_rows", "one_launch", "fused_tile",
    "estage_union"};

}  // namespace

// Device start/stop events of the kernels of the steps it is handed to (lsh_decode_step_timed).
struct lsh_profiler {
    int max_launches = 0;
    std::vector<hipEvent_t> ev[LSH_NUM_KERNELS];  // start/stop pairs
    int used[LSH_NUM_KERNELS] = {0, 0, 0, 0, 0};
};

struct lsh_tables {
    int device = 0;
    const void* E = nullptr;
    int V = 0, d = 0, dtype = 0, K = 0, P = 0, W = 0, u = 0, bits = 0;
    int64_t ld = 0;
    int32_t* perms_dev = nullptr;    // [P, K]
    int32_t* codes_dev = nullptr;    // [V, W] band codes of the embedding rows
    int32_t* words_dev = nullptr;    // [W, V] word ids grouped by band code
    Slot* slots_dev = nullptr;       // all bands' cuckoo slots, concatenated
    uint4* cuts_dev = nullptr;       // per slot: where vocabulary slices 1..3 begin in its span
    BandMeta* bands_dev = nullptr;   // [W]
    std::vector<HostBand> bands;
    int wg_candidates_lds = 0;
    int wg_fused_lds = 0;
    int wg_hit_rows_lds = 0;   // 0: the hit-count kernel cannot run on these tables (t > 1 unsupported)
    int hit_list_cap = 0;
    int wg_union_logits_lds = 0;
    int built_on_device = 0, build_attempts = 0;  // how the tables came about (inspection)
    void* scratch_dev = nullptr;                  // this device's copy of the static scratch array
    // Ticket counters of the one-launch plan: kTicketSlots blocks of kTicketBlock counters in
    // device memory, all zero between steps (the kernel that uses a block leaves it zero).  A
    // block belongs to one workspace address for the life of the handle, so steps that run at the
    // same time -- which must use different workspaces -- never share counters.  The table is a
    // cache behind the const handle: guarded by its own mutex, it changes no result.
    unsigned int* tickets_dev = nullptr;
    mutable std::mutex ticket_mu;
    mutable const void* ticket_owner[kTicketSlots] = {};
    mutable int ticket_used = 0;
    // The counters for the step that works in `workspace`, or null when all blocks are taken (the
    // step then ends with a selection kernel of its own).
    unsigned int* tickets_for(const void* workspace) const {
        std::lock_guard<std::mutex> lock(ticket_mu);
        for (int i = 0; i < ticket_used; ++i)
            if (ticket_owner[i] == workspace) return tickets_dev + (size_t)i * kTicketBlock;
        if (!tickets_dev || ticket_used == kTicketSlots) return nullptr;
        ticket_owner[ticket_used] = workspace;
        return tickets_dev + (size_t)(ticket_used++) * kTicketBlock;
    }
    int opt[kNumOpts];                            // launch-plan options, kAuto unless set
    int option(int which, int dflt) const { return opt[which] == kAuto ? dflt : opt[which]; }
};

namespace {

struct SplitMix64 {
    uint64_t s;
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

inline int code_bits(int K) {
    int b = 0;
    while ((1 << b) < K) ++b;
    return b;
}

// Two-choice cuckoo insertion (Pagh & Rodler) of the band's keys into `cap` slots.  Returns false
// if some insertion exceeds the eviction limit with these hash parameters.
bool cuckoo_try(const HostBand& hb, const BandMeta& m, int cap, Slot* slots) {
    for (int i = 0; i < cap; ++i) slots[i] = Slot{-1, 0u, 0u, 0u};
    int lg = 0;
    while ((1 << lg) < cap) ++lg;
    const int max_kicks = 16 * (lg + 1);
    for (size_t q = 0; q < hb.keys.size(); ++q) {
        Slot cur{hb.keys[q], (uint32_t)hb.offsets[q], (uint32_t)(hb.offsets[q + 1] - hb.offsets[q]), 0u};
        const uint32_t h0 = cuckoo_hash(m.a0, m.b0, (uint32_t)cur.key, m.shift);
        const uint32_t h1 = cuckoo_hash(m.a1, m.b1, (uint32_t)cur.key, m.shift);
        bool placed = false;
        if (slots[h0].key < 0) { slots[h0] = cur; placed = true; }
        else if (slots[h1].key < 0) { slots[h1] = cur; placed = true; }
        uint32_t pos = h0;
        for (int kick = 0; !placed && kick < max_kicks; ++kick) {
            // take slot `pos`; its occupant moves to its own other slot, evicting in turn
            std::swap(cur, slots[pos]);
            const uint32_t e0 = cuckoo_hash(m.a0, m.b0, (uint32_t)cur.key, m.shift);
            const uint32_t e1 = cuckoo_hash(m.a1, m.b1, (uint32_t)cur.key, m.shift);
            pos = (pos == e0) ? e1 : e0;
            if (slots[pos].key < 0) { slots[pos] = cur; placed = true; }
        }
        if (!placed) return false;
    }
    return true;
}

lsh_status build_cuckoo(HostBand& hb, SplitMix64& rng, std::vector<Slot>& out, uint32_t slot_off) {
    int cap = 2;
    while ((size_t)cap < 2 * hb.keys.size()) cap <<= 1;
    std::vector<Slot> slots;
    for (int grow = 0; grow < 4; ++grow, cap <<= 1) {
        slots.resize(cap);
        int lg = 0;
        while ((1 << lg) < cap) ++lg;
        for (int attempt = 0; attempt < 16; ++attempt) {
            BandMeta m{};
            m.slot_off = slot_off;
            m.shift = 32u - (uint32_t)lg;
            m.a0 = (uint32_t)rng.next() | 1u;
            m.b0 = (uint32_t)rng.next();
            m.a1 = (uint32_t)rng.next() | 1u;
            m.b1 = (uint32_t)rng.next();
            if (cuckoo_try(hb, m, cap, slots.data())) {
                hb.capacity = cap;
                hb.meta = m;
                out.insert(out.end(), slots.begin(), slots.end());
                return LSH_OK;
            }
        }
    }
    return LSH_ERR_BUILD_FAILED;
}

// What a step's launches share: the (read-only) tables, the stream, and the caller's profiler.
struct StepCtx {
    const lsh_tables* t;
    hipStream_t st;
    lsh_profiler* prof;
};

template <typename... KArgs, typename... Args>
void launch(const StepCtx& cx, int which, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem,
            Args... args) {
    lsh_profiler* pf = cx.prof;
    hipStream_t stream = cx.st;
    if (pf && which >= 0 && pf->used[which] < pf->max_launches) {
        const int i = pf->used[which]++;
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)shmem, stream, pf->ev[which][2 * i],
                              pf->ev[which][2 * i + 1], 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)shmem, stream, args...);
    }
}

Workspace carve(const lsh_tables* t, const lsh_step_params* sp, void* base) {
    return carve_workspace(sp->S, sp->B, t->V, sp->full_vocab != 0, base);
}

bool step_params_ok(const lsh_tables* t, const lsh_step_params* sp) {
    return t && sp && sp->S >= 1 && sp->B >= 1 && sp->B <= kMaxB && sp->T >= 0 &&
           sp->S <= kMaxSentencesLogits && (int64_t)sp->S * sp->B <= (int64_t)INT32_MAX / 2;
}

int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : dflt;
}

// Raises a kernel's dynamic-LDS limit to (nearly) a CU's whole LDS, once per kernel and device.
// The limit belongs to the kernel, not to a table: it is never set to what one table needs, and
// the decode step makes no driver call besides its launches once a kernel has been through here.
template <auto KFN>
hipError_t allow_whole_lds() {
    static std::atomic<uint64_t> done{0};  // one bit per device
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0ull;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute((const void*)KFN, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxDynLds);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// Little work per step (few sentences x 16-row groups): every workgroup of the logits grid
// regenerates the candidates itself (k_cand_logits); otherwise one candidates workgroup per
// sentence, then the logits grid.  LSHBEAM_FUSED=0/1 overrides the size rule (for tests and
// measurements), never the hard limits.
bool step_is_fused(const lsh_tables* t, const lsh_step_params* sp) {
    const int MT = (sp->B + kTileM - 1) / kTileM;
    const bool possible = !sp->full_vocab && (size_t)t->wg_fused_lds <= kMaxDynLds && sp->S <= 64;
    // (with three or more groups of 16 beams the separate split-k kernel, one (tile, group) per
    // workgroup at a time, is faster than the fused kernel's all-groups-per-tile loop)
    const bool wanted = t->option(kOptFused, (sp->S * MT <= 8 && MT <= 2) ? 1 : 0) != 0;
    return possible && wanted;
}

// LDS words for the staged hidden rows of a step: room for all B rows of a sentence (up to
// kCandStageRows; LSHBEAM_STAGE_ROWS overrides, 0 = never more than the minimum) where LDS has
// it beside everything else the kernel keeps there, else the minimum stage.
int stage_words_for(const lsh_tables* t, int B, bool fused_kernel) {
    const int mn = candidates_min_stage(t->d);
    const int rows = std::min(B, std::max(0, t->option(kOptStageRows, kCandStageRows)));
    const int64_t want = ((int64_t)rows * t->d + 3) & ~(int64_t)3;
    const size_t other = fused_kernel ? fused_lds_words(t->V, t->P, t->K, 0)
                                      : candidates_lds_words(t->V, t->P, t->K, 0);
    const size_t room = kMaxDynLds / sizeof(uint32_t);
    const int64_t cap = room > other ? (int64_t)((room - other) & ~(size_t)3) : 0;
    return (int)std::max<int64_t>(mn, std::min(want, cap));
}

// Rows of a sentence hashed per workgroup when the sentence is cut into parts (t = 1, more beams
// than one chunk of hashing holds even with the step's stage); 0 = the sentence is hashed by one
// workgroup.  Parts take the minimum stage.  LSHBEAM_PART_ROWS forces a part size (for tests and
// measurements).
int part_rows_of(const lsh_tables* t, const lsh_step_params* sp, int stage_words) {
    if (sp->full_vocab || sp->threshold != 1) return 0;
    const int rpc = candidates_rows_per_chunk(sp->B, t->d, t->W, candidates_min_stage(t->d));
    const int forced = t->option(kOptPartRows, 0);
    if (forced > 0) return std::min(forced, rpc);
    return sp->B > candidates_rows_per_chunk(sp->B, t->d, t->W, stage_words) ? rpc : 0;
}

template <typename ET, int WAVES>
void launch_logits_w(const StepCtx& cx, int grid, bool aligned, const float* H,
                     const lsh_step_params* sp, const int32_t* cand, const int32_t* count,
                     const Workspace& w) {
    const lsh_tables* t = cx.t;
    constexpr int UNROLL = (WAVES >= 16) ? 4 : 8;
    const ET* E = (const ET*)t->E;
    if (aligned)
        launch(cx, 1, k_logits<ET, WAVES, UNROLL, true>, dim3(grid), dim3(WAVES * kWave), 0, E,
               t->ld, t->d, H, sp->S, sp->B, cand, count, t->V, w.logits, w.cpitch, w.records());
    else
        launch(cx, 1, k_logits<ET, WAVES, UNROLL, false>, dim3(grid), dim3(WAVES * kWave), 0, E,
               t->ld, t->d, H, sp->S, sp->B, cand, count, t->V, w.logits, w.cpitch, w.records());
}

template <typename ET, int MT>
void launch_logits_wave(const StepCtx& cx, int grid, bool aligned, const float* H,
                        const lsh_step_params* sp, const int32_t* cand, const int32_t* count,
                        const Workspace& w) {
    const lsh_tables* t = cx.t;
    // loads in flight per lane: 32 (fp32) / 64 (bf16) bytes of E per step, plus MT times that of H
    constexpr int UNROLL = ((MT == 1) ? 8 : 4) / (ElemTraits<ET>::VEC / 4);
    const ET* E = (const ET*)t->E;
    if (aligned)
        launch(cx, 1, k_logits_wave<ET, MT, UNROLL, true>, dim3(grid), dim3(256), 0, E, t->ld, t->d,
               H, sp->S, sp->B, cand, count, t->V, w.logits, w.cpitch, w.records());
    else
        launch(cx, 1, k_logits_wave<ET, MT, UNROLL, false>, dim3(grid), dim3(256), 0, E, t->ld, t->d,
               H, sp->S, sp->B, cand, count, t->V, w.logits, w.cpitch, w.records());
}

// k_logits_hlds over the sentence's rows in groups: a group's rows must fit in LDS.  Up to 78 KB
// two 8-wave workgroups share a CU, beyond that one 16-wave workgroup has it alone.  Returns 0
// if even one 16-row group does not fit (very large d): the caller then keeps the hidden rows
// in global memory.
constexpr size_t kHldsHalf = 78 * 1024;
inline int hlds_group_rows(const lsh_tables* t, int S, int B, int d) {
    const int forced = t->option(kOptHldsRows, 0);  // 16 or 32 (measurements)
    if (forced == 16 || forced == 32)
        return hlds_lds_bytes(S, std::min(forced, B), d, 16) <= kMaxDynLds ? std::min(forced, B) : 0;
    // up to 32 beams: one group; more: groups of 16, a workgroup each (measured at S = 4: B = 50,
    // V = 100k: 51 us with groups of 16, 46 with 32, 55 with the rows in global memory; B = 48,
    // V = 40k: 48 / 54 / 51)
    if (B > 32) return hlds_lds_bytes(S, 16, d, 16) <= kMaxDynLds ? 16 : 0;
    for (int rows : {32, 16})
        if (hlds_lds_bytes(S, std::min(rows, B), d, 16) <= kMaxDynLds) return std::min(rows, B);
    return 0;
}

template <typename ET>
void launch_logits_hlds(const StepCtx& cx, int64_t tiles_n, bool aligned, const float* H,
                        const lsh_step_params* sp, const int32_t* cand, const int32_t* count,
                        const Workspace& w, int group_rows) {
    const lsh_tables* t = cx.t;
    constexpr int U1 = 8 / (ElemTraits<ET>::VEC / 4), U2 = 4 / (ElemTraits<ET>::VEC / 4);
    // (1024-thread workgroups have 128 registers per lane: one load less in flight)
    constexpr int U2W = (U2 > 2) ? U2 - 1 : U2;
    const ET* E = (const ET*)t->E;
    // one launch: a workgroup serves one group of `rows` hidden rows (the last group may be smaller)
    const int rows = std::min(group_rows, sp->B);
    const int ngroups = (sp->B + rows - 1) / rows;
#define LSH_HLDS(MTV, WV, UV, AL, PL)                                                                \
    do {                                                                                             \
        auto kfn = k_logits_hlds<ET, MTV, WV, UV, AL, PL>;                                           \
        const size_t lds = hlds_lds_bytes(sp->S, rows, t->d, WV, PL);                                \
        const int gx = (int)std::min<int64_t>(                                                       \
            tiles_n, std::max(1, t->option(kOptLogitsGrid, 4096 / WV) / ngroups));              \
        const int grid = ((gx + 7) / 8 * 8) * ngroups;                                               \
        launch(cx, 1, kfn, dim3(grid), dim3(WV * kWave), lds, E, t->ld, t->d, H, sp->S, sp->B,   \
               rows, gx, ngroups, t->option(kOptHldsRem, 4), cand, count, t->V, w.logits,      \
               w.cpitch, w.records());                                                      \
    } while (0)
    // bf16 rows, up to 16 hidden rows per group, two workgroups per CU: the hidden rows go to LDS
    // as three bf16 planes and the contraction runs on bf16 matrix instructions
    // (LSHBEAM_LOGITS_PLANES=0: widened to fp32 as for every other shape)
    if constexpr (std::is_same<ET, uint16_t>::value) {
        if (aligned && rows <= kTileM && hlds_lds_bytes(sp->S, rows, t->d, 8, true) <= kHldsHalf &&
            t->option(kOptLogitsPlanes, 1)) {
            LSH_HLDS(1, 8, U1, true, true);
            return;
        }
    }
    const bool two = rows > kTileM;
    const bool small = hlds_lds_bytes(sp->S, rows, t->d, 8) <= kHldsHalf;
    if (small) {
        if (two) { if (aligned) LSH_HLDS(2, 8, U2, true, false); else LSH_HLDS(2, 8, U2, false, false); }
        else { if (aligned) LSH_HLDS(1, 8, U1, true, false); else LSH_HLDS(1, 8, U1, false, false); }
    } else {
        if (two) { if (aligned) LSH_HLDS(2, 16, U2W, true, false); else LSH_HLDS(2, 16, U2W, false, false); }
        else { if (aligned) LSH_HLDS(1, 16, U1, true, false); else LSH_HLDS(1, 16, U1, false, false); }
    }
#undef LSH_HLDS
}

// k_logits_estage: 33..64 beams, fp32 rows of at most 1024 values, 16-byte aligned operands, at
// most 256 sentences.  About one workgroup per CU, dealt evenly to the sentences.
// Returns its workgroups per sentence: each leaves one record per hidden row for all its tiles.
// un, if given: the kernel makes the candidate list itself, from the bitmaps of the sentence's parts.
int launch_logits_estage(const StepCtx& cx, const float* H, const lsh_step_params* sp,
                         const int32_t* cand, const int32_t* count, const Workspace& w,
                         const EstageUnion* un = nullptr) {
    const lsh_tables* t = cx.t;
    const float* E = (const float*)t->E;
    const int MT = (sp->B + kTileM - 1) / kTileM;
    const size_t lds = estage_lds_bytes(un != nullptr);
    const int per_sentence = std::max(1, t->option(kOptLogitsGrid, 256) / sp->S);
    const dim3 grid((unsigned)(per_sentence * sp->S)), block(1024);
#define LSH_ESTAGE(MTV, UN)                                                                          \
    do {                                                                                             \
        auto kfn = k_logits_estage<MTV, UN>;                                                         \
        launch(cx, 1, kfn, grid, block, lds, E, t->ld, t->d, H, sp->S, sp->B, cand, count, t->V,     \
               w.logits, w.cpitch, w.records(), un ? *un : EstageUnion{});                           \
    } while (0)
    if (un) { if (MT <= 3) LSH_ESTAGE(3, true); else LSH_ESTAGE(4, true); }
    else { if (MT <= 3) LSH_ESTAGE(3, false); else LSH_ESTAGE(4, false); }
#undef LSH_ESTAGE
    return per_sentence;
}

// Whether a step's contraction is k_logits_estage: 33..64 beams, fp32 rows of at most 1024 values,
// 16-byte aligned operands, at most 256 sentences (option logits_estage = 0: the other drivers).
bool takes_estage(const lsh_tables* t, const lsh_step_params* sp, const float* H) {
    const bool aligned = (t->d % 4 == 0) && (t->ld % 4 == 0) && ((uintptr_t)t->E % 16 == 0) && ((uintptr_t)H % 16 == 0);
    return t->dtype == LSH_F32 && aligned && sp->B > 2 * kTileM && sp->B <= 4 * kTileM &&
           t->d <= kEsSlices * kEsSlice && sp->S <= 256 && estage_lds_bytes(true) <= kMaxDynLds &&
           t->option(kOptLogitsEstage, 1) && !t->option(kOptLogitsWaves, 0);
}

// Returns 0 if the kernel it launched leaves one record per hidden row and tile, else the number
// of record groups per sentence (see select_sentence).
template <typename ET>
int launch_logits(const StepCtx& cx, const float* H, const lsh_step_params* sp,
                  const int32_t* cand, const int32_t* count, const Workspace& w,
                  const EstageUnion* un = nullptr) {
    const lsh_tables* t = cx.t;
    constexpr int VEC = ElemTraits<ET>::VEC;
    const bool aligned = (t->d % VEC == 0) && (t->ld % VEC == 0) && ((uintptr_t)t->E % 16 == 0) &&
                         (t->d % 4 == 0) && ((uintptr_t)H % 16 == 0);
    const int MT = (sp->B + kTileM - 1) / kTileM;
    const int64_t tiles_n = (int64_t)sp->S * ((t->V + kTileN - 1) / kTileN);  // upper bound
    const int64_t max_tiles = tiles_n * MT;
    // Few (sentence, M-tile) groups: little work per step and it is latency that counts, so k is
    // split across the 16 waves of a workgroup and the partial tiles are summed through LDS.
    // Otherwise one wave per 16-candidate tile, no LDS and no barrier (up to 4 M-tiles per wave).
    // (the full-vocabulary mode has V / 16 tiles per sentence, known here: thousands of tiles
    // are "many" even for one sentence -- 29.9 against 37.1 us at V = 40000)
    const bool few = sp->S * MT <= 8 && !(count == nullptr && tiles_n >= 1024);
    const int mode = t->option(kOptLogitsWaves, few ? 16 : 1);
    // one wave per tile with the sentence's hidden rows staged in LDS, more than 32 rows in
    // groups; LSHBEAM_LOGITS_HLDS=0 keeps the rows in global memory (k_logits_wave)
    const int group_rows = hlds_group_rows(t, sp->S, sp->B, t->d);
    // 33..64 beams: hidden rows in registers, candidate rows through LDS (LSHBEAM_LOGITS_ESTAGE=0:
    // the other drivers)
    if (takes_estage(t, sp, H)) {
        return launch_logits_estage(cx, H, sp, cand, count, w, un);
    } else if (mode == 1 && group_rows > 0 && t->option(kOptLogitsHlds, 1)) {
        launch_logits_hlds<ET>(cx, tiles_n, aligned, H, sp, cand, count, w, group_rows);
    } else if (mode == 1 && MT <= 4) {
        const int grid = (int)std::min<int64_t>((tiles_n + 3) / 4, t->option(kOptLogitsGrid, 1024));
        switch (MT) {
            case 1: launch_logits_wave<ET, 1>(cx, grid, aligned, H, sp, cand, count, w); break;
            case 2: launch_logits_wave<ET, 2>(cx, grid, aligned, H, sp, cand, count, w); break;
            case 3: launch_logits_wave<ET, 3>(cx, grid, aligned, H, sp, cand, count, w); break;
            default: launch_logits_wave<ET, 4>(cx, grid, aligned, H, sp, cand, count, w); break;
        }
    } else if (mode >= 16) {
        const int grid = (int)std::min<int64_t>(max_tiles, t->option(kOptLogitsGrid, 256));
        launch_logits_w<ET, 16>(cx, grid, aligned, H, sp, cand, count, w);
    } else {
        const int grid = (int)std::min<int64_t>(max_tiles, t->option(kOptLogitsGrid, 2048));
        launch_logits_w<ET, 4>(cx, grid, aligned, H, sp, cand, count, w);
    }
    return 0;
}

template <typename ET>
hipError_t allow_logits_lds() {
    constexpr int U1 = 8 / (ElemTraits<ET>::VEC / 4), U2 = 4 / (ElemTraits<ET>::VEC / 4);
    constexpr int U2W = (U2 > 2) ? U2 - 1 : U2;
    hipError_t e = hipSuccess;
#define LSH_ALLOW(...)                                                   \
    do {                                                                 \
        if (e == hipSuccess) e = allow_whole_lds<k_logits_hlds<ET, __VA_ARGS__>>(); \
    } while (0)
    LSH_ALLOW(1, 8, U1, true, false);  LSH_ALLOW(1, 8, U1, false, false);
    LSH_ALLOW(2, 8, U2, true, false);  LSH_ALLOW(2, 8, U2, false, false);
    LSH_ALLOW(1, 16, U1, true, false); LSH_ALLOW(1, 16, U1, false, false);
    LSH_ALLOW(2, 16, U2W, true, false); LSH_ALLOW(2, 16, U2W, false, false);
    if constexpr (std::is_same<ET, uint16_t>::value) LSH_ALLOW(1, 8, U1, true, true);
#undef LSH_ALLOW
    return e;
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            (void)hipGetLastError();                    \
            return e_ == hipErrorOutOfMemory ? LSH_ERR_OOM : LSH_ERR_HIP; \
        }                                               \
    } while (0)

// Host path of the table build: codes are copied back, every band's (code, id) pairs are sorted
// and inserted into its cuckoo table on the host, then uploaded.
lsh_status build_on_host(lsh_tables* t, hipStream_t st, SplitMix64& rng) {
    const size_t V = t->V, W = t->W;
    (void)hipFree(t->words_dev); t->words_dev = nullptr;
    (void)hipFree(t->slots_dev); t->slots_dev = nullptr;
    (void)hipFree(t->cuts_dev); t->cuts_dev = nullptr;
    (void)hipFree(t->bands_dev); t->bands_dev = nullptr;
    t->bands.clear();
    std::vector<Slot> slots_host;
    std::vector<int32_t> codes(V * W);
    HIP_TRY(hipMemcpyAsync(codes.data(), t->codes_dev, V * W * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));

    // per band: group word ids by code (ids ascending inside a span), then the cuckoo table
    std::vector<int32_t> words(V * W);
    std::vector<uint64_t> order(V);
    t->bands.resize(W);
    for (size_t w = 0; w < W; ++w) {
        for (size_t j = 0; j < V; ++j)
            order[j] = ((uint64_t)(uint32_t)codes[j * W + w] << 32) | (uint64_t)j;
        std::sort(order.begin(), order.end());
        HostBand& hb = t->bands[w];
        for (size_t i = 0; i < V; ++i) {
            const int32_t code = (int32_t)(order[i] >> 32);
            if (i == 0 || code != hb.keys.back()) {
                hb.keys.push_back(code);
                hb.offsets.push_back((int32_t)i);
            }
            words[w * V + i] = (int32_t)(uint32_t)order[i];
        }
        hb.offsets.push_back((int32_t)V);
        const lsh_status rc = build_cuckoo(hb, rng, slots_host, (uint32_t)slots_host.size());
        if (rc != LSH_OK) return rc;
    }
    std::vector<BandMeta> metas(W);
    for (size_t w = 0; w < W; ++w) metas[w] = t->bands[w].meta;

    // 16 bytes of slack: k_hit_rows reads ids with 16-byte loads that may straddle the end
    HIP_TRY(hipMalloc((void**)&t->words_dev, V * W * sizeof(int32_t) + 16));
    // where the vocabulary slices of the hit-count kernel begin inside every span
    std::vector<uint4> cuts_host(slots_host.size(), make_uint4(0u, 0u, 0u, 0u));
    const int slice_ids = hit_slice_words(t->V);
    for (size_t w = 0; w < W; ++w) {
        const BandMeta& m = t->bands[w].meta;
        for (int i = 0; i < t->bands[w].capacity; ++i) {
            const Slot& sl = slots_host[m.slot_off + i];
            if (sl.key < 0) continue;
            const int32_t* span = words.data() + w * V + sl.start;
            uint32_t c[3];
            for (int q = 1; q <= 3; ++q)
                c[q - 1] = (uint32_t)(std::lower_bound(span, span + sl.len, q * slice_ids) - span);
            cuts_host[m.slot_off + i] = make_uint4(c[0], c[1], c[2], sl.len);
        }
    }
    HIP_TRY(hipMalloc((void**)&t->cuts_dev, cuts_host.size() * sizeof(uint4)));
    HIP_TRY(hipMemcpyAsync(t->cuts_dev, cuts_host.data(), cuts_host.size() * sizeof(uint4),
                           hipMemcpyHostToDevice, st));
    HIP_TRY(hipMalloc((void**)&t->slots_dev, slots_host.size() * sizeof(Slot)));
    HIP_TRY(hipMalloc((void**)&t->bands_dev, W * sizeof(BandMeta)));
    HIP_TRY(hipMemcpyAsync(t->words_dev, words.data(), V * W * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(t->slots_dev, slots_host.data(), slots_host.size() * sizeof(Slot),
                           hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(t->bands_dev, metas.data(), W * sizeof(BandMeta), hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));

    return LSH_OK;
}

struct DevBuf {  // temporary device memory of the build, released on every exit path
    void* p = nullptr;
    ~DevBuf() { (void)hipFree(p); }
    template <typename T> T* as() const { return (T*)p; }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
};

inline int bits_for(uint64_t max_value) {  // bits needed to write max_value (at least 1)
    int b = 1;
    while (b < 64 && (max_value >> b)) ++b;
    return b;
}

// Device path of the table build (build_tables.h).  LSH_ERR_BUILD_FAILED = some band could not
// be inserted after all attempts (or the problem is too large for the 32-bit item counts of the
// sort): the caller falls back to the host path.
lsh_status build_on_device(lsh_tables* t, hipStream_t st, SplitMix64& rng) {
    const int64_t V = t->V, W = t->W, N = V * W;
    if (N >= (int64_t)INT32_MAX) return LSH_ERR_BUILD_FAILED;
    const SortKeyLayout lay{bits_for((uint64_t)V - 1), std::max(1, t->u * t->bits)};
    const int key_bits = lay.id_bits + lay.code_bits + bits_for((uint64_t)W - 1);
    const dim3 blk(256), grdN((unsigned)((N + 255) / 256));

    DevBuf keys_a, keys_b, head, key_index, tmp;
    HIP_TRY(keys_a.alloc(N * sizeof(uint64_t)));
    HIP_TRY(keys_b.alloc(N * sizeof(uint64_t)));
    HIP_TRY(head.alloc(N * sizeof(uint32_t)));
    HIP_TRY(key_index.alloc(N * sizeof(uint32_t)));
    hipLaunchKernelGGL(k_make_sort_keys, grdN, blk, 0, st, (const int32_t*)t->codes_dev, V, (int)W, lay,
                       keys_a.as<uint64_t>());
    size_t sort_bytes = 0, scan_bytes = 0;
    HIP_TRY(hipcub::DeviceRadixSort::SortKeys(nullptr, sort_bytes, keys_a.as<uint64_t>(),
                                              keys_b.as<uint64_t>(), (int)N, 0, key_bits, st));
    HIP_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, scan_bytes, head.as<uint32_t>(),
                                             key_index.as<uint32_t>(), (int)N, st));
    HIP_TRY(tmp.alloc(std::max(sort_bytes, scan_bytes)));
    HIP_TRY(hipcub::DeviceRadixSort::SortKeys(tmp.p, sort_bytes, keys_a.as<uint64_t>(),
                                              keys_b.as<uint64_t>(), (int)N, 0, key_bits, st));
    // 16 bytes of slack: k_hit_rows reads ids with 16-byte loads that may straddle the end
    HIP_TRY(hipMalloc((void**)&t->words_dev, N * sizeof(int32_t) + 16));
    hipLaunchKernelGGL(k_split_sorted, grdN, blk, 0, st, (const uint64_t*)keys_b.p, V, (int)W, lay,
                       t->words_dev, head.as<uint32_t>());
    HIP_TRY(hipcub::DeviceScan::ExclusiveSum(tmp.p, scan_bytes, head.as<uint32_t>(),
                                             key_index.as<uint32_t>(), (int)N, st));
    // keys per band: the scan value at each band's first position, and the total
    std::vector<uint32_t> first_key(W + 1);
    uint32_t last_index = 0, last_head = 0;
    HIP_TRY(hipMemcpy2DAsync(first_key.data(), sizeof(uint32_t), key_index.p, (size_t)V * sizeof(uint32_t),
                             sizeof(uint32_t), (size_t)W, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&last_index, key_index.as<uint32_t>() + (N - 1), sizeof(uint32_t),
                           hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&last_head, head.as<uint32_t>() + (N - 1), sizeof(uint32_t),
                           hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    const uint32_t n_keys = last_index + last_head;
    first_key[W] = n_keys;

    DevBuf key_code, key_start, key_band, key_len;
    HIP_TRY(key_code.alloc(n_keys * sizeof(int32_t)));
    HIP_TRY(key_start.alloc(n_keys * sizeof(uint32_t)));
    HIP_TRY(key_band.alloc(n_keys * sizeof(int32_t)));
    HIP_TRY(key_len.alloc(n_keys * sizeof(uint32_t)));
    hipLaunchKernelGGL(k_emit_keys, grdN, blk, 0, st, (const uint64_t*)keys_b.p, (const uint32_t*)head.p,
                       (const uint32_t*)key_index.p, V, (int)W, lay, key_code.as<int32_t>(),
                       key_start.as<uint32_t>(), key_band.as<int32_t>());
    const dim3 grdK((n_keys + 255) / 256);
    hipLaunchKernelGGL(k_key_lengths, grdK, blk, 0, st, (const uint32_t*)key_start.p,
                       (const int32_t*)key_band.p, n_keys, (uint32_t)V, key_len.as<uint32_t>());
    DevBuf key_cut;
    HIP_TRY(key_cut.alloc(n_keys * sizeof(uint4)));
    hipLaunchKernelGGL(k_slice_cuts, grdK, blk, 0, st, (const int32_t*)t->words_dev,
                       (const uint32_t*)key_start.p, (const uint32_t*)key_len.p, (const int32_t*)key_band.p,
                       n_keys, (uint32_t)V, hit_slice_words(t->V), key_cut.as<uint4>());

    // table geometry: a power of two of at least three slots per key and band (load <= 1/3:
    // two-choice cuckoo insertion then succeeds at the first attempt almost always)
    t->bands.assign(W, HostBand{});
    std::vector<BandMeta> metas(W);
    std::vector<uint32_t> caps(W), flags(W, 0u);
    uint64_t n_slots = 0;
    int max_lg = 1;
    for (int64_t w = 0; w < W; ++w) {
        const uint32_t nk = first_key[w + 1] - first_key[w];
        int lg = 1;
        while ((uint64_t)(1u << lg) < 3ull * nk) ++lg;
        max_lg = std::max(max_lg, lg);
        caps[w] = 1u << lg;
        metas[w] = BandMeta{};
        metas[w].slot_off = (uint32_t)n_slots;
        metas[w].shift = 32u - (uint32_t)lg;
        n_slots += caps[w];
    }
    if (n_slots >= (1ull << 32)) return LSH_ERR_BUILD_FAILED;
    auto draw = [&](BandMeta& m) {
        m.a0 = (uint32_t)rng.next() | 1u; m.b0 = (uint32_t)rng.next();
        m.a1 = (uint32_t)rng.next() | 1u; m.b1 = (uint32_t)rng.next();
    };
    for (auto& m : metas) draw(m);

    DevBuf table, caps_dev, redo_dev, failed_dev;
    HIP_TRY(table.alloc(n_slots * sizeof(uint64_t)));
    HIP_TRY(caps_dev.alloc(W * sizeof(uint32_t)));
    HIP_TRY(redo_dev.alloc(W * sizeof(uint32_t)));
    HIP_TRY(failed_dev.alloc(W * sizeof(uint32_t)));
    HIP_TRY(hipMalloc((void**)&t->bands_dev, W * sizeof(BandMeta)));
    HIP_TRY(hipMalloc((void**)&t->slots_dev, n_slots * sizeof(Slot)));
    HIP_TRY(hipMalloc((void**)&t->cuts_dev, n_slots * sizeof(uint4)));
    HIP_TRY(hipMemcpyAsync(caps_dev.p, caps.data(), W * sizeof(uint32_t), hipMemcpyHostToDevice, st));
    const dim3 grdClear((unsigned)std::min<uint64_t>(64, ((1ull << max_lg) + 255) / 256), (unsigned)W);
    // LSHBEAM_CUCKOO_CHAIN shortens the eviction chains (tests of the retry and fallback paths)
    const int max_chain = env_int("LSHBEAM_CUCKOO_CHAIN", 16 * (max_lg + 1));
    bool done = false;
    for (int attempt = 0; attempt < 24 && !done; ++attempt) {
        t->build_attempts = attempt + 1;
        const uint32_t* redo = attempt ? redo_dev.as<uint32_t>() : nullptr;
        HIP_TRY(hipMemcpyAsync(t->bands_dev, metas.data(), W * sizeof(BandMeta), hipMemcpyHostToDevice, st));
        HIP_TRY(hipMemsetAsync(failed_dev.p, 0, W * sizeof(uint32_t), st));
        hipLaunchKernelGGL(k_cuckoo_clear, grdClear, blk, 0, st, table.as<uint64_t>(),
                           (const BandMeta*)t->bands_dev, (const uint32_t*)caps_dev.p, (int)W, redo);
        if (n_keys)
            hipLaunchKernelGGL(k_cuckoo_insert, grdK, blk, 0, st, table.as<uint64_t>(),
                               (const BandMeta*)t->bands_dev, (const int32_t*)key_code.p,
                               (const int32_t*)key_band.p, n_keys, max_chain, redo,
                               failed_dev.as<uint32_t>());
        HIP_TRY(hipMemcpyAsync(flags.data(), failed_dev.p, W * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        done = true;
        for (int64_t w = 0; w < W; ++w)
            if (flags[w]) { done = false; draw(metas[w]); }
        if (!done)
            HIP_TRY(hipMemcpyAsync(redo_dev.p, flags.data(), W * sizeof(uint32_t), hipMemcpyHostToDevice, st));
    }
    if (!done) return LSH_ERR_BUILD_FAILED;
    hipLaunchKernelGGL(k_cuckoo_finalize, dim3((unsigned)((n_slots + 255) / 256)), blk, 0, st,
                       (const uint64_t*)table.p, n_slots, (const uint32_t*)key_start.p,
                       (const uint32_t*)key_len.p, (const uint4*)key_cut.p, t->slots_dev, t->cuts_dev);
    HIP_TRY(hipGetLastError());

    // host mirrors for the inspection calls: distinct codes and span boundaries of every band
    std::vector<int32_t> codes_h(n_keys);
    std::vector<uint32_t> starts_h(n_keys);
    HIP_TRY(hipMemcpyAsync(codes_h.data(), key_code.p, n_keys * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(starts_h.data(), key_start.p, n_keys * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int64_t w = 0; w < W; ++w) {
        HostBand& hb = t->bands[w];
        hb.keys.assign(codes_h.begin() + first_key[w], codes_h.begin() + first_key[w + 1]);
        hb.offsets.assign(starts_h.begin() + first_key[w], starts_h.begin() + first_key[w + 1]);
        hb.offsets.push_back((int32_t)V);
        hb.capacity = (int)caps[w];
        hb.meta = metas[w];
    }
    t->built_on_device = 1;
    return LSH_OK;
}

// The decode step behind every public variant of it: validation, launch plan, launches.
lsh_status decode_step_impl(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                            const int32_t* topfreq_dev, const lsh_step_params* sp,
                            void* workspace_dev, size_t workspace_bytes, int32_t* out_beam_dev,
                            int32_t* out_word_dev, float* out_score_dev, void* hip_stream,
                            lsh_profiler* prof) {
    if (!t || !H_dev || !beam_scores_dev || !sp || !workspace_dev || !out_beam_dev ||
        !out_word_dev || !out_score_dev)
        return LSH_ERR_INVALID_ARG;
    if (!step_params_ok(t, sp)) return LSH_ERR_INVALID_ARG;
    if (!sp->full_vocab && sp->T > 0 && !topfreq_dev) return LSH_ERR_INVALID_ARG;
    if (!sp->full_vocab && sp->threshold < 1) return LSH_ERR_INVALID_ARG;
    if (!sp->full_vocab && sp->threshold > 1 && t->wg_hit_rows_lds == 0) return LSH_ERR_UNSUPPORTED;
    if ((uintptr_t)workspace_dev % kAlign) return LSH_ERR_INVALID_ARG;
    const Workspace w = carve(t, sp, workspace_dev);
    if (workspace_bytes < w.bytes) return LSH_ERR_WORKSPACE_TOO_SMALL;
    const StepCtx cx{t, (hipStream_t)hip_stream, prof};
    const int32_t* cand = nullptr;
    const int32_t* count = nullptr;
    const bool fused = step_is_fused(t, sp);
    const int stage = stage_words_for(t, sp->B, fused);
    CandArgs ca{H_dev, sp->B, t->d, t->perms_dev, t->P, t->K, t->W, t->bits, t->slots_dev,
                t->bands_dev, t->words_dev, t->V, topfreq_dev, sp->T, t->cuts_dev, stage};
    set_derived(ca);
    // Bitmaps made by an earlier kernel, to be OR-ed per sentence: one per hidden row when the
    // hit threshold is above 1 (Eq. 9-10), one per part of the sentence when it has many beams.
    const uint32_t* parts = nullptr;
    int nparts = 0;
    if (!sp->full_vocab && sp->threshold > 1) {
        launch(cx, 3, k_hit_rows, dim3(sp->S * sp->B * kHitSlices), dim3(kCandThreads), (size_t)t->wg_hit_rows_lds,
               ca, (int)sp->threshold, t->hit_list_cap, w.row_bitmaps);
        parts = w.row_bitmaps;
        nparts = sp->B;
    } else if (const int pr = part_rows_of(t, sp, stage)) {
        nparts = (sp->B + pr - 1) / pr;
        ca.stage_words = candidates_min_stage(t->d);
        set_derived(ca);
        launch(cx, 4, k_part_bitmaps, dim3(sp->S * nparts), dim3(kCandThreads), (size_t)t->wg_candidates_lds,
               ca, pr, nparts, w.row_bitmaps);
        parts = w.row_bitmaps;
    }
    bool selected = false;   // the step's tail already ran inside the fused kernel
    int rec_groups = 0;      // tile records per hidden row, if not one per tile (launch_logits)
    if (fused) {
        // One launch per step: the last workgroup of each sentence also runs the selection
        // (option one_launch = 0: a selection kernel follows instead; also when no ticket block
        // is left for this workspace or the step has more sentences than a block has counters).
        TailArgs tail{nullptr, beam_scores_dev, w.lse, out_beam_dev, out_word_dev, out_score_dev,
                      std::max(0, t->option(kOptFusedTile, 0))};
        if (t->option(kOptOneLaunch, 0) && sp->S <= kTicketBlock) tail.tickets = t->tickets_for(workspace_dev);
        selected = tail.tickets != nullptr;
        const int per_sentence = std::min(kMaxFusedGrid, std::max(1, t->option(kOptFusedGrid, 256) / sp->S));
        const dim3 grid((unsigned)(per_sentence * sp->S)), block(kCandThreads);
        const bool aligned16 = ((uintptr_t)t->E % 16 == 0) && (t->d % 4 == 0) && ((uintptr_t)H_dev % 16 == 0);
        const bool f32 = t->dtype == LSH_F32;
        const bool al = f32 ? (aligned16 && t->ld % 4 == 0) : (aligned16 && t->ld % 8 == 0 && t->d % 8 == 0);
        if (parts) {
            const size_t lds = (size_t)t->wg_union_logits_lds;
#define LSH_UNION_LOGITS(ET, AL, OL)                                                              \
    launch(cx, 1, k_union_logits<ET, AL, OL>, grid, block, lds, parts, nparts, topfreq_dev, sp->T, \
           (const ET*)t->E, t->ld, t->d, H_dev, sp->S, sp->B, t->V, w.cand, w.count, w.logits,    \
           w.cpitch, w.records(), tail)
#define LSH_UNION_LOGITS2(ET, AL) \
    do { if (selected) LSH_UNION_LOGITS(ET, AL, true); else LSH_UNION_LOGITS(ET, AL, false); } while (0)
            if (f32) { if (al) LSH_UNION_LOGITS2(float, true); else LSH_UNION_LOGITS2(float, false); }
            else { if (al) LSH_UNION_LOGITS2(uint16_t, true); else LSH_UNION_LOGITS2(uint16_t, false); }
#undef LSH_UNION_LOGITS2
#undef LSH_UNION_LOGITS
        } else {
            const size_t lds = fused_lds_words(t->V, t->P, t->K, stage) * sizeof(uint32_t);
#define LSH_CAND_LOGITS(ET, AL, OL)                                                               \
    launch(cx, 1, k_cand_logits<ET, AL, OL>, grid, block, lds, ca, (const ET*)t->E, t->ld, sp->S,  \
           w.cand, w.count, w.logits, w.cpitch, w.records(), tail)
#define LSH_CAND_LOGITS2(ET, AL) \
    do { if (selected) LSH_CAND_LOGITS(ET, AL, true); else LSH_CAND_LOGITS(ET, AL, false); } while (0)
            if (f32) { if (al) LSH_CAND_LOGITS2(float, true); else LSH_CAND_LOGITS2(float, false); }
            else { if (al) LSH_CAND_LOGITS2(uint16_t, true); else LSH_CAND_LOGITS2(uint16_t, false); }
#undef LSH_CAND_LOGITS2
#undef LSH_CAND_LOGITS
        }
        cand = w.cand;
        count = w.count;
    } else {
        // a few part bitmaps ahead of k_logits_estage: that kernel ORs them itself (option
        // estage_union = 0: a union kernel of its own, as for the other drivers)
        EstageUnion un{parts, nparts, topfreq_dev, sp->T, w.cand, w.count};
        const bool fold = parts && nparts <= kEsUnionParts && takes_estage(t, sp, H_dev) && t->option(kOptEstageUnion, 1) &&
                          estage_union_words(t->V) <= (size_t)2 * kTileN * kEsPitch;
        if (fold) {
            cand = w.cand;
            count = w.count;
        } else if (parts) {
            // union of the sentence's bitmaps + top-frequent words + compaction
            launch(cx, 0, k_union_compact, dim3(sp->S), dim3(kCandThreads),
                   union_compact_lds_words(t->V) * sizeof(uint32_t), parts, nparts, t->V,
                   topfreq_dev, sp->T, w.cand, w.count);
            cand = w.cand;
            count = w.count;
        } else if (!sp->full_vocab) {
            launch(cx, 0, k_candidates, dim3(sp->S), dim3(kCandThreads),
                   candidates_lds_words(t->V, t->P, t->K, stage) * sizeof(uint32_t), ca, w.cand, w.count);
            cand = w.cand;
            count = w.count;
        }
        rec_groups = t->dtype == LSH_F32 ? launch_logits<float>(cx, H_dev, sp, cand, count, w, fold ? &un : nullptr)
                                         : launch_logits<uint16_t>(cx, H_dev, sp, cand, count, w);
    }
    if (!selected) {
#define LSH_SELECT(RICHV, GROUPSV)                                                                    \
    launch(cx, 2, k_select<RICHV, GROUPSV>, dim3(sp->S), dim3(kSelThreads), 0, (const float*)w.logits,  \
           w.cpitch, (const TileRecord*)w.partials, (const int32_t*)w.ids2, w.ppitch, cand, count, t->V, \
           sp->B, beam_scores_dev, w.lse, out_beam_dev, out_word_dev, out_score_dev,                   \
           fused ? std::max(0, t->option(kOptFusedTile, 0)) : 0, rec_groups)
        // (the fused kernels leave rich records, k_logits_estage one record for a group of tiles)
        if (fused) LSH_SELECT(true, false); else if (rec_groups > 0) LSH_SELECT(false, true); else LSH_SELECT(false, false);
#undef LSH_SELECT
    }
    HIP_TRY(hipGetLastError());
    return LSH_OK;
}

}  // namespace

extern "C" {

const char* lsh_status_string(lsh_status s) {
    switch (s) {
        case LSH_OK: return "ok";
        case LSH_ERR_INVALID_ARG: return "invalid argument";
        case LSH_ERR_UNSUPPORTED: return "unsupported parameter";
        case LSH_ERR_BUILD_FAILED: return "cuckoo table build failed";
        case LSH_ERR_OOM: return "out of device memory";
        case LSH_ERR_HIP: return "HIP runtime error";
        case LSH_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case LSH_ERR_SCRATCH_TOO_SMALL: return "step too large for the built-in scratch buffer";
    }
    return "unknown status";
}

int32_t lsh_step_is_fused(const lsh_tables* t, const lsh_step_params* sp) {
    return (step_params_ok(t, sp) && step_is_fused(t, sp)) ? 1 : 0;
}

const char* lsh_kernel_name(int32_t which) {
    switch (which) {
        case 0: return "k_candidates";
        case 1: return "k_logits";
        case 2: return "k_select";
        case 3: return "k_hit_rows";
        case 4: return "k_part_bitmaps";
    }
    return "";
}

void lsh_free_tables(lsh_tables* t) {
    if (!t) return;
    (void)hipFree(t->perms_dev);
    (void)hipFree(t->codes_dev);
    (void)hipFree(t->words_dev);
    (void)hipFree(t->slots_dev);
    (void)hipFree(t->cuts_dev);
    (void)hipFree(t->bands_dev);
    (void)hipFree(t->tickets_dev);
    delete t;
}

lsh_status lsh_build_tables(const void* E_dev, const int32_t* perms_dev, const lsh_build_params* p,
                            void* hip_stream, lsh_tables** out) {
    if (!E_dev || !perms_dev || !p || !out) return LSH_ERR_INVALID_ARG;
    *out = nullptr;
    if (p->V < 1 || p->V > kMaxV || p->d < 1 || p->ld_e < p->d) return LSH_ERR_INVALID_ARG;
    if (p->e_dtype != LSH_F32 && p->e_dtype != LSH_BF16) return LSH_ERR_INVALID_ARG;
    if (p->K < 2 || p->K > p->d || p->K > 32768) return LSH_ERR_INVALID_ARG;
    if (p->P < 1 || p->bands < 1 || p->P % p->bands != 0) return LSH_ERR_INVALID_ARG;
    const int bits = code_bits(p->K), u = p->P / p->bands;
    if ((int64_t)u * bits > 30) return LSH_ERR_INVALID_ARG;
    if (candidates_lds_words(p->V, p->P, p->K, candidates_min_stage(p->d)) * 4 > kMaxDynLds ||
        p->bands > kCandThreads)
        return LSH_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)hip_stream;

    lsh_tables* t = new (std::nothrow) lsh_tables();
    if (!t) return LSH_ERR_OOM;
    struct Guard { lsh_tables* t; ~Guard() { if (t) lsh_free_tables(t); } } guard{t};
    HIP_TRY(hipGetDevice(&t->device));
    HIP_TRY(scratch_of_device(t->device, &t->scratch_dev));
    HIP_TRY(hipMalloc((void**)&t->tickets_dev, (size_t)kTicketSlots * kTicketBlock * sizeof(unsigned int)));
    HIP_TRY(hipMemsetAsync(t->tickets_dev, 0, (size_t)kTicketSlots * kTicketBlock * sizeof(unsigned int),
                           (hipStream_t)hip_stream));
    // launch-plan options: the library's own rules unless LSHBEAM_<NAME> is set in the environment
    // at this point (read once, here) or lsh_set_option changes them later
    for (int i = 0; i < kNumOpts; ++i) {
        std::string name = "LSHBEAM_";
        for (const char* c = kOptNames[i]; *c; ++c) name += (char)std::toupper((unsigned char)*c);
        t->opt[i] = env_int(name.c_str(), kAuto);
    }
    t->E = E_dev; t->V = p->V; t->d = p->d; t->ld = p->ld_e; t->dtype = p->e_dtype;
    t->K = p->K; t->P = p->P; t->W = p->bands; t->u = u; t->bits = bits;
    const size_t V = t->V, W = t->W, PK = (size_t)t->P * t->K;

    // permutations: copy, validate on the host
    std::vector<int32_t> perms(PK);
    HIP_TRY(hipMemcpyAsync(perms.data(), perms_dev, PK * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int32_t x : perms)
        if (x < 0 || x >= t->d) return LSH_ERR_INVALID_ARG;
    HIP_TRY(hipMalloc((void**)&t->perms_dev, PK * sizeof(int32_t)));
    HIP_TRY(hipMemcpyAsync(t->perms_dev, perms.data(), PK * sizeof(int32_t), hipMemcpyHostToDevice, st));

    // band codes of every embedding row, on the device
    HIP_TRY(hipMalloc((void**)&t->codes_dev, V * W * sizeof(int32_t)));
    {
        const int64_t n = (int64_t)V * W;
        const dim3 grid((unsigned)((n + 255) / 256)), block(256);
        if (t->dtype == LSH_F32)
            hipLaunchKernelGGL(k_band_codes<float>, grid, block, 0, st, (const float*)E_dev, t->ld,
                               (int64_t)V, t->perms_dev, t->P, t->K, t->W, bits, t->codes_dev);
        else
            hipLaunchKernelGGL(k_band_codes<uint16_t>, grid, block, 0, st, (const uint16_t*)E_dev,
                               t->ld, (int64_t)V, t->perms_dev, t->P, t->K, t->W, bits, t->codes_dev);
        HIP_TRY(hipGetLastError());
    }
    // bucket tables + cuckoo tables: on the device; LSHBEAM_HOST_BUILD=1 (tests) or a band that
    // keeps failing its insertion takes the host path instead
    SplitMix64 rng{p->seed ^ 0xC0FFEE1234ABCDEFull};
    lsh_status brc = env_int("LSHBEAM_HOST_BUILD", 0) ? LSH_ERR_BUILD_FAILED : build_on_device(t, st, rng);
    if (brc == LSH_ERR_BUILD_FAILED) brc = build_on_host(t, st, rng);
    if (brc != LSH_OK) return brc;

    // (with the minimum stage; a step may ask for more)
    t->wg_candidates_lds = (int)(candidates_lds_words(t->V, t->P, t->K, candidates_min_stage(t->d)) * sizeof(uint32_t));
    {   // LDS plan of k_hit_rows: whatever the counters leave goes to the load list
        const size_t fixed = hit_rows_fixed_lds_words(t->V, t->d, t->P);
        const size_t room = kMaxDynLds / sizeof(uint32_t);
        size_t cap = room > fixed ? (room - fixed) / 1024 * 1024 : 0;
        if (cap > (size_t)kHitListMax) cap = kHitListMax;
        if (cap >= (size_t)kHitListMin && (uint64_t)t->W * (uint64_t)t->V < (1ull << 30)) {
            t->hit_list_cap = (int)cap;
            t->wg_hit_rows_lds = (int)((fixed + cap) * sizeof(uint32_t));
        }
    }
    t->wg_union_logits_lds = (int)(union_logits_lds_words(t->V) * sizeof(uint32_t));
    t->wg_fused_lds = (int)(fused_lds_words(t->V, t->P, t->K, candidates_min_stage(t->d)) * sizeof(uint32_t));
    HIP_TRY(allow_whole_lds<k_candidates>());
    HIP_TRY(allow_whole_lds<k_hit_rows>());
    HIP_TRY(allow_whole_lds<k_union_compact>());
    HIP_TRY(allow_whole_lds<k_part_bitmaps>());
#define LSH_ALLOW_FUSED(ET, AL)                                          \
    HIP_TRY((allow_whole_lds<k_union_logits<ET, AL, false>>()));         \
    HIP_TRY((allow_whole_lds<k_union_logits<ET, AL, true>>()));          \
    HIP_TRY((allow_whole_lds<k_cand_logits<ET, AL, false>>()));          \
    HIP_TRY((allow_whole_lds<k_cand_logits<ET, AL, true>>()))
    LSH_ALLOW_FUSED(float, true);
    LSH_ALLOW_FUSED(float, false);
    LSH_ALLOW_FUSED(uint16_t, true);
    LSH_ALLOW_FUSED(uint16_t, false);
#undef LSH_ALLOW_FUSED
    HIP_TRY(allow_logits_lds<float>());
    HIP_TRY(allow_logits_lds<uint16_t>());
    HIP_TRY((allow_whole_lds<k_logits_estage<3, false>>()));
    HIP_TRY((allow_whole_lds<k_logits_estage<4, false>>()));
    HIP_TRY((allow_whole_lds<k_logits_estage<3, true>>()));
    HIP_TRY((allow_whole_lds<k_logits_estage<4, true>>()));
    guard.t = nullptr;
    *out = t;
    return LSH_OK;
}

size_t lsh_step_workspace_bytes(const lsh_tables* t, const lsh_step_params* sp) {
    if (!step_params_ok(t, sp)) return 0;
    return carve(t, sp, nullptr).bytes;
}

lsh_status lsh_decode_step(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                           const int32_t* topfreq_dev, const lsh_step_params* sp,
                           void* workspace_dev, size_t workspace_bytes, int32_t* out_beam_dev,
                           int32_t* out_word_dev, float* out_score_dev, void* hip_stream) {
    return decode_step_impl(t, H_dev, beam_scores_dev, topfreq_dev, sp, workspace_dev, workspace_bytes,
                            out_beam_dev, out_word_dev, out_score_dev, hip_stream, nullptr);
}

lsh_status lsh_decode_step_timed(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                                 const int32_t* topfreq_dev, const lsh_step_params* sp,
                                 void* workspace_dev, size_t workspace_bytes, int32_t* out_beam_dev,
                                 int32_t* out_word_dev, float* out_score_dev, void* hip_stream,
                                 lsh_profiler* prof) {
    return decode_step_impl(t, H_dev, beam_scores_dev, topfreq_dev, sp, workspace_dev, workspace_bytes,
                            out_beam_dev, out_word_dev, out_score_dev, hip_stream, prof);
}

size_t lsh_static_scratch_bytes(void) { return kScratchBytes; }

lsh_status lsh_decode_step_static(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                                  const int32_t* topfreq_dev, const lsh_step_params* sp,
                                  int32_t* out_beam_dev, int32_t* out_word_dev, float* out_score_dev,
                                  void* hip_stream) {
    if (!step_params_ok(t, sp)) return LSH_ERR_INVALID_ARG;
    if (!t->scratch_dev) return LSH_ERR_HIP;
    if (carve(t, sp, nullptr).bytes > kScratchBytes) return LSH_ERR_SCRATCH_TOO_SMALL;
    // (nothing in the workspace has to start from zero: every kernel writes what a later one reads)
    return decode_step_impl(t, H_dev, beam_scores_dev, topfreq_dev, sp, t->scratch_dev, kScratchBytes,
                            out_beam_dev, out_word_dev, out_score_dev, hip_stream, nullptr);
}

lsh_status lsh_set_option(lsh_tables* t, const char* name, int32_t value) {
    if (!t || !name || value < kAuto) return LSH_ERR_INVALID_ARG;
    for (int i = 0; i < kNumOpts; ++i)
        if (std::strcmp(name, kOptNames[i]) == 0) { t->opt[i] = value; return LSH_OK; }
    return LSH_ERR_INVALID_ARG;
}

lsh_status lsh_get_option(const lsh_tables* t, const char* name, int32_t* value_out) {
    if (!t || !name || !value_out) return LSH_ERR_INVALID_ARG;
    for (int i = 0; i < kNumOpts; ++i)
        if (std::strcmp(name, kOptNames[i]) == 0) { *value_out = t->opt[i]; return LSH_OK; }
    return LSH_ERR_INVALID_ARG;
}

/* ---- inspection ----------------------------------------------------------------------------- */

lsh_status lsh_debug_codes(const lsh_tables* t, const float* H_dev, int32_t R, int32_t* codes_host) {
    if (!t || !H_dev || !codes_host || R < 1) return LSH_ERR_INVALID_ARG;
    int32_t* tmp = nullptr;
    const int64_t n = (int64_t)R * t->W;
    HIP_TRY(hipMalloc((void**)&tmp, n * sizeof(int32_t)));
    hipLaunchKernelGGL(k_band_codes<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, 0, H_dev,
                       (int64_t)t->d, (int64_t)R, (const int32_t*)t->perms_dev, t->P, t->K, t->W,
                       t->bits, tmp);
    hipError_t e = hipMemcpy(codes_host, tmp, n * sizeof(int32_t), hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    HIP_TRY(e);
    return LSH_OK;
}

lsh_status lsh_debug_embedding_codes(const lsh_tables* t, int32_t row0, int32_t n, int32_t* codes_host) {
    if (!t || !codes_host || row0 < 0 || n < 0 || (int64_t)row0 + n > t->V) return LSH_ERR_INVALID_ARG;
    HIP_TRY(hipMemcpy(codes_host, t->codes_dev + (size_t)row0 * t->W, (size_t)n * t->W * sizeof(int32_t),
                      hipMemcpyDeviceToHost));
    return LSH_OK;
}

lsh_status lsh_debug_bucket(const lsh_tables* t, int32_t band, int32_t code, int32_t* words_host,
                            int32_t cap, int32_t* n_out) {
    if (!t || !n_out || band < 0 || band >= t->W || cap < 0 || (cap > 0 && !words_host))
        return LSH_ERR_INVALID_ARG;
    // read the two slots the device would read, from device memory
    const BandMeta& m = t->bands[band].meta;
    *n_out = -1;
    if (code < 0) return LSH_OK;
    const uint32_t h[2] = {cuckoo_hash(m.a0, m.b0, (uint32_t)code, m.shift),
                           cuckoo_hash(m.a1, m.b1, (uint32_t)code, m.shift)};
    for (int q = 0; q < 2; ++q) {
        Slot sl;
        HIP_TRY(hipMemcpy(&sl, t->slots_dev + m.slot_off + h[q], sizeof(Slot), hipMemcpyDeviceToHost));
        if (sl.key == code) {
            *n_out = (int32_t)sl.len;
            const size_t ncopy = std::min<size_t>(sl.len, (size_t)cap);
            if (ncopy)
                HIP_TRY(hipMemcpy(words_host, t->words_dev + (size_t)band * t->V + sl.start,
                                  ncopy * sizeof(int32_t), hipMemcpyDeviceToHost));
            return LSH_OK;
        }
    }
    return LSH_OK;
}

lsh_status lsh_debug_csr(const lsh_tables* t, int32_t band, int32_t* n_keys_out, int32_t* keys_host,
                         int32_t* offsets_host, int32_t cap_keys, int32_t* words_host) {
    if (!t || band < 0 || band >= t->W || !n_keys_out) return LSH_ERR_INVALID_ARG;
    const HostBand& hb = t->bands[band];
    *n_keys_out = (int32_t)hb.keys.size();
    if (keys_host && offsets_host && cap_keys >= (int32_t)hb.keys.size()) {
        std::memcpy(keys_host, hb.keys.data(), hb.keys.size() * sizeof(int32_t));
        std::memcpy(offsets_host, hb.offsets.data(), hb.offsets.size() * sizeof(int32_t));
    }
    if (words_host)
        HIP_TRY(hipMemcpy(words_host, t->words_dev + (size_t)band * t->V, (size_t)t->V * sizeof(int32_t),
                          hipMemcpyDeviceToHost));
    return LSH_OK;
}

lsh_status lsh_debug_build_info(const lsh_tables* t, int32_t* on_device_out, int32_t* attempts_out) {
    if (!t || !on_device_out || !attempts_out) return LSH_ERR_INVALID_ARG;
    *on_device_out = t->built_on_device;
    *attempts_out = t->build_attempts;
    return LSH_OK;
}

lsh_status lsh_debug_cuckoo_shape(const lsh_tables* t, int32_t band, int32_t* capacity_out,
                                  int32_t* n_keys_out) {
    if (!t || band < 0 || band >= t->W || !capacity_out || !n_keys_out) return LSH_ERR_INVALID_ARG;
    *capacity_out = t->bands[band].capacity;
    *n_keys_out = (int32_t)t->bands[band].keys.size();
    return LSH_OK;
}

lsh_status lsh_debug_candidates(const lsh_tables* t, const void* workspace_dev,
                                const lsh_step_params* sp, int32_t s, int32_t* cand_host,
                                int32_t cap, int32_t* n_out) {
    if (!t || !workspace_dev || !n_out || !step_params_ok(t, sp) || sp->full_vocab || s < 0 ||
        s >= sp->S || cap < 0 || (cap > 0 && !cand_host))
        return LSH_ERR_INVALID_ARG;
    const Workspace w = carve(t, sp, const_cast<void*>(workspace_dev));
    HIP_TRY(hipDeviceSynchronize());
    int32_t n = 0;
    HIP_TRY(hipMemcpy(&n, w.count + s, sizeof(int32_t), hipMemcpyDeviceToHost));
    *n_out = n;
    const size_t ncopy = (size_t)std::min(n, cap);
    if (ncopy)
        HIP_TRY(hipMemcpy(cand_host, w.cand + (size_t)s * t->V, ncopy * sizeof(int32_t),
                          hipMemcpyDeviceToHost));
    return LSH_OK;
}

lsh_status lsh_debug_counts(const lsh_tables* t, const void* workspace_dev, const lsh_step_params* sp,
                            int32_t* counts_host) {
    if (!t || !workspace_dev || !counts_host || !step_params_ok(t, sp)) return LSH_ERR_INVALID_ARG;
    if (sp->full_vocab) {
        for (int s = 0; s < sp->S; ++s) counts_host[s] = t->V;
        return LSH_OK;
    }
    const Workspace w = carve(t, sp, const_cast<void*>(workspace_dev));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(counts_host, w.count, (size_t)sp->S * sizeof(int32_t), hipMemcpyDeviceToHost));
    return LSH_OK;
}

lsh_status lsh_debug_logprobs(const lsh_tables* t, const void* workspace_dev,
                              const lsh_step_params* sp, int32_t s, float* lp_host, int32_t cap,
                              int32_t* n_out) {
    if (!t || !workspace_dev || !n_out || !lp_host || !step_params_ok(t, sp) || s < 0 ||
        s >= sp->S || cap < 1)
        return LSH_ERR_INVALID_ARG;
    const Workspace w = carve(t, sp, const_cast<void*>(workspace_dev));
    HIP_TRY(hipDeviceSynchronize());
    int32_t C = t->V;
    if (!sp->full_vocab) HIP_TRY(hipMemcpy(&C, w.count + s, sizeof(int32_t), hipMemcpyDeviceToHost));
    *n_out = C;
    const int n = std::min(C, cap);
    if (n == 0) return LSH_OK;
    float* tmp = nullptr;
    HIP_TRY(hipMalloc((void**)&tmp, (size_t)sp->B * cap * sizeof(float)));
    hipLaunchKernelGGL(k_logprobs_dump, dim3((unsigned)((n + 255) / 256), (unsigned)sp->B), dim3(256), 0,
                       0, (const float*)w.logits, w.cpitch, (const float*)w.lse, s * sp->B, sp->B, n,
                       tmp, (int64_t)cap);
    hipError_t e = hipMemcpy(lp_host, tmp, (size_t)sp->B * cap * sizeof(float), hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    HIP_TRY(e);
    return LSH_OK;
}

/* ---- per-kernel timing ---------------------------------------------------------------------- */

void lsh_profiler_destroy(lsh_profiler* pf) {
    if (!pf) return;
    for (int k = 0; k < LSH_NUM_KERNELS; ++k)
        for (hipEvent_t e : pf->ev[k]) (void)hipEventDestroy(e);
    delete pf;
}

lsh_status lsh_profiler_create(int32_t max_launches, lsh_profiler** out) {
    if (!out || max_launches < 1 || max_launches > (1 << 16)) return LSH_ERR_INVALID_ARG;
    *out = nullptr;
    lsh_profiler* pf = new (std::nothrow) lsh_profiler();
    if (!pf) return LSH_ERR_OOM;
    pf->max_launches = max_launches;
    for (int k = 0; k < LSH_NUM_KERNELS; ++k)
        for (int i = 0; i < 2 * max_launches; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) {
                (void)hipGetLastError();
                lsh_profiler_destroy(pf);
                return LSH_ERR_HIP;
            }
            pf->ev[k].push_back(e);
        }
    *out = pf;
    return LSH_OK;
}

lsh_status lsh_profiler_read(lsh_profiler* pf, double mean_ms_out[LSH_NUM_KERNELS],
                             int32_t launches_out[LSH_NUM_KERNELS]) {
    if (!pf || !mean_ms_out || !launches_out) return LSH_ERR_INVALID_ARG;
    HIP_TRY(hipDeviceSynchronize());
    for (int k = 0; k < LSH_NUM_KERNELS; ++k) {
        double total = 0.0;
        for (int i = 0; i < pf->used[k]; ++i) {
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, pf->ev[k][2 * i], pf->ev[k][2 * i + 1]));
            total += ms;
        }
        launches_out[k] = pf->used[k];
        mean_ms_out[k] = pf->used[k] ? total / pf->used[k] : 0.0;
        pf->used[k] = 0;
    }
    return LSH_OK;
}

lsh_status lsh_beam_advance(const lsh_beam_params* bp, int32_t step, const int32_t* out_beam_dev,
                            const int32_t* out_word_dev, const float* out_score_dev,
                            const float* const* states_in, float* const* states_out,
                            int32_t* backptr_dev, int32_t* words_dev, float* scores_dev,
                            float* next_scores_dev, void* hip_stream) {
    if (!bp || !out_beam_dev || !out_word_dev || !out_score_dev || !backptr_dev || !words_dev ||
        !scores_dev || !next_scores_dev)
        return LSH_ERR_INVALID_ARG;
    if (bp->S < 1 || bp->B < 1 || bp->B > kMaxB || (int64_t)bp->S * bp->B > INT32_MAX / 2 ||
        bp->n_states < 0 || bp->n_states > kMaxBeamStates || bp->max_len < 1 || step < 0 ||
        step >= bp->max_len || (bp->n_states > 0 && (bp->state_dim < 1 || !states_in || !states_out)))
        return LSH_ERR_INVALID_ARG;
    BeamStatePtrs ptrs{};
    for (int k = 0; k < bp->n_states; ++k) {
        if (!states_in[k] || !states_out[k] || states_in[k] == states_out[k]) return LSH_ERR_INVALID_ARG;
        ptrs.in[k] = states_in[k];
        ptrs.out[k] = states_out[k];
    }
    const size_t R = (size_t)bp->S * bp->B, off = (size_t)step * R;
    hipLaunchKernelGGL(k_beam_advance, dim3((unsigned)R, (unsigned)std::max(bp->n_states, 1)), dim3(256), 0,
                       (hipStream_t)hip_stream, ptrs, (int)bp->n_states, (int)bp->state_dim, (int)bp->B,
                       (int)bp->eos, out_beam_dev, out_word_dev, out_score_dev, backptr_dev + off,
                       words_dev + off, scores_dev + off, next_scores_dev);
    HIP_TRY(hipGetLastError());
    return LSH_OK;
}

lsh_status lsh_beam_backtrace(const lsh_beam_params* bp, int32_t n_steps, const int32_t* backptr_dev,
                              const int32_t* words_dev, const float* scores_dev, int32_t* tokens_dev,
                              int32_t* length_dev, float* best_score_dev, void* hip_stream) {
    if (!bp || !backptr_dev || !words_dev || !scores_dev || !tokens_dev || !length_dev || !best_score_dev)
        return LSH_ERR_INVALID_ARG;
    if (bp->S < 1 || bp->B < 1 || bp->B > kMaxB || bp->max_len < 1 || n_steps < 0 ||
        n_steps > bp->max_len || (int64_t)n_steps * bp->B > INT32_MAX / 2)
        return LSH_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_beam_backtrace, dim3((unsigned)bp->S), dim3(kWave), 0, (hipStream_t)hip_stream,
                       (int)bp->S, (int)bp->B, (int)bp->eos, (int)n_steps, backptr_dev, words_dev,
                       scores_dev, (int)bp->max_len, tokens_dev, length_dev, best_score_dev);
    HIP_TRY(hipGetLastError());
    return LSH_OK;
}

}  // extern "C"
