/* lshbeam -- LSH reduced-vocabulary softmax + beam expansion on one MI355X (gfx950).
 *
 * C ABI of the decode-time hot path of Shi, Xu & Knight, "Fast Locality Sensitive Hashing for
 * Beam Search on GPU":  winner-take-all hashing of the hidden states (Eq. 4-8), lookup of the
 * band codes in per-band cuckoo tables (section "Cuckoo lookup", Algorithm 1), the candidate
 * list shared across a sentence's beams and merged with the top-frequent words (Eq. 3, Eq. 10),
 * the gathered product H * E_LSH (Eq. 2), the log-softmax over the candidate list (Eq. 1) and
 * the beam expansion (Introduction, "Beam expansion") -- all on the device.
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; *_host is host memory.
 *  - The library allocates device memory only inside lsh_build_tables (freed by
 *    lsh_free_tables).  lsh_decode_step allocates nothing, works in a caller workspace, is
 *    asynchronous on the given HIP stream and performs no host synchronisation and no
 *    device-to-host copy.
 *  - Errors are return codes; arguments are validated on the host before any launch and a
 *    failed call leaves the outputs untouched.  No C++ exception crosses this boundary.
 *  - All calls on one lsh_tables must be made with the device it was built on current.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - Word ids and beam ids are 0-based; a beam id is the row index inside its sentence.
 */
#ifndef LSHBEAM_H
#define LSHBEAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lsh_tables lsh_tables; /* opaque; owns the device tables */

typedef enum {
    LSH_OK = 0,
    LSH_ERR_INVALID_ARG = 1,
    LSH_ERR_UNSUPPORTED = 2,
    LSH_ERR_BUILD_FAILED = 3,
    LSH_ERR_OOM = 4,
    LSH_ERR_HIP = 5,
    LSH_ERR_WORKSPACE_TOO_SMALL = 6,
    LSH_ERR_SCRATCH_TOO_SMALL = 7 /* lsh_decode_step_static: the step needs more than the built-in buffer */
} lsh_status;

typedef enum { LSH_F32 = 0, LSH_BF16 = 1 } lsh_dtype;

/* The paper's hash hyper-parameters {K, u, W} (text after Eq. 8) plus the layout of E. */
typedef struct {
    int32_t V;       /* vocabulary size = rows of E, 1 .. 2^24                                   */
    int32_t d;       /* hidden size = columns of E                                               */
    int64_t ld_e;    /* row pitch of E in elements, >= d                                         */
    int32_t e_dtype; /* lsh_dtype: fp32, or bf16 bit patterns                                    */
    int32_t K;       /* WTA window: each code is the argmax over K permuted dims, 2 <= K <= d    */
    int32_t P;       /* number of permutations = codes per vector                                */
    int32_t bands;   /* W; P % W == 0; u = P / W codes per band; u * ceil(log2 K) <= 30          */
    uint64_t seed;   /* seeds the cuckoo hash functions only (results never depend on it)        */
} lsh_build_params;

/* Build the index over the rows of E (once, after training, or again whenever E changes; section
 * "Cuckoo lookup", first step).
 *   E_dev      [V, ld_e] row-major, fp32 or bf16.  BORROWED: must stay valid and unchanged until
 *              lsh_free_tables; the decode step gathers its rows.
 *   perms_dev  int32 [P, K]: row p holds the first K entries of permutation p of 0..d-1
 *              (Eq. 5: Permute_p(x)[k] = x[perms[p][k]]).  Copied; validated to lie in [0, d).
 * Computes the band code of every row on the device (ties in the argmax go to the lowest k),
 * groups word ids by band code into one flat array per band (ids ascending inside a span; one
 * device radix sort over all bands) and stores (start, length) of every span in a two-choice
 * cuckoo table per band (parallel insertion on the device; the host only draws the hash
 * parameters and takes over if a band cannot be placed).
 * Synchronous.  On success *out receives the handle. */
lsh_status lsh_build_tables(const void* E_dev, const int32_t* perms_dev, const lsh_build_params* p,
                            void* hip_stream, lsh_tables** out);

void lsh_free_tables(lsh_tables* t); /* NULL-safe */

/* Per-call shape of a decode step; the paper's remaining hyper-parameters {B, T, t}. */
typedef struct {
    int32_t S;          /* sentences in the call; hidden rows R = S * B                          */
    int32_t B;          /* beams per sentence, 1 .. 256; also the number of results per sentence */
    int32_t T;          /* length of the top-frequent word list (may be 0)                       */
    int32_t threshold;  /* t of Eq. 10, >= 1: a word is a candidate iff some row of the sentence
                           shares at least t band codes with it.  t > 1 keeps a quarter of a row
                           of 16-bit hit counters in LDS: LSH_ERR_UNSUPPORTED if V is too large
                           for that (about 290000 words) or bands * V >= 2^30                  */
    int32_t full_vocab; /* 1: skip hashing, the candidate list is all of V (Eq. 1-2 as printed)  */
} lsh_step_params;

/* Bytes of workspace lsh_decode_step needs for these parameters (0 on invalid arguments). */
size_t lsh_step_workspace_bytes(const lsh_tables* t, const lsh_step_params* sp);

/* One decode step for S sentences of B beams.
 *   H_dev            fp32 [S*B, d], pitch d: top-layer hidden states, sentence-major.
 *   beam_scores_dev  fp32 [S*B]: accumulated log-probability of each beam (-inf = dead beam).
 *   topfreq_dev      int32 [T]: ids of the top-frequent words V_T (Eq. 3); ids outside [0, V)
 *                    are ignored; duplicates are harmless.
 *   workspace_dev    >= lsh_step_workspace_bytes() bytes, 256-byte aligned; contents need not be
 *                    initialised and are overwritten.  Two steps that overlap in time must not
 *                    share a workspace.
 * Per sentence s: V_LSH,s = V_T U { j : some row of s shares a band code with E_j } in ascending
 * id order; logit = H_s * E[V_LSH,s]^T accumulated in fp32; log-probabilities normalised over
 * V_LSH,s; the B best (beam, word) pairs by beam_score + log-probability, best first, equal
 * scores ordered by lower beam then lower word id.
 *   out_beam_dev / out_word_dev / out_score_dev   [S, B].  If fewer than B pairs have a finite
 *   score the tail is (-1, -1, -inf). */
lsh_status lsh_decode_step(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                           const int32_t* topfreq_dev, const lsh_step_params* sp,
                           void* workspace_dev, size_t workspace_bytes, int32_t* out_beam_dev,
                           int32_t* out_word_dev, float* out_score_dev, void* hip_stream);

/* The decode step for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as lsh_decode_step, but the working memory is a buffer built into the
 * library: a static device array of lsh_static_scratch_bytes() = 32 MiB that every GPU the library
 * runs on holds until the process ends (its address on a GPU is looked up once, when the first
 * handle is built there).  The call allocates and frees nothing, on the device or through any
 * allocating library routine.
 *   - LSH_ERR_SCRATCH_TOO_SMALL if lsh_step_workspace_bytes(t, sp) exceeds the buffer (V = 40000:
 *     about 150 hidden rows per call); nothing is launched and the outputs are untouched.
 *   - All calls on one GPU share that GPU's buffer, across handles and streams: calls that overlap
 *     in time race.  Serialise them (one stream, or events), or give lsh_decode_step workspaces.
 *   - The buffer keeps the last call's contents; no step depends on them (every kernel of a step
 *     writes what a later kernel of the same step reads). */
size_t lsh_static_scratch_bytes(void);
lsh_status lsh_decode_step_static(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                                  const int32_t* topfreq_dev, const lsh_step_params* sp,
                                  int32_t* out_beam_dev, int32_t* out_word_dev, float* out_score_dev,
                                  void* hip_stream);

/* ---- beam bookkeeping around the step (Introduction, "Beam expansion"; Table 1, row "Hidden
 *      states reorder") ----------------------------------------------------------------------- */

typedef struct {
    int32_t S, B;      /* as in lsh_step_params                                                   */
    int32_t n_states;  /* recurrent state arrays reordered per step, 0 .. 16 (a 2-layer LSTM: 4)  */
    int32_t state_dim; /* fp32 values per row of every state array                                */
    int32_t eos;       /* word id that ends a hypothesis, or -1 for none                          */
    int32_t max_len;   /* time steps the history arrays hold                                      */
} lsh_beam_params;

/* After lsh_decode_step at time step `step` (0-based): slot b of sentence s continues parent beam
 * p = out_beam[s, b] with word w = out_word[s, b].  For every state array k:
 *   states_out[k][s*B + b, :] = states_in[k][s*B + p, :]   (zeros for an empty slot, p = -1);
 * the choice is recorded, backptr[step, s, b] = p, words[step, s, b] = w, scores[step, s, b] =
 * out_score[s, b]; and the accumulated scores for the next step are written:
 *   next_scores[s, b] = out_score[s, b], or -inf if w == eos or the slot is empty
 * (a finished hypothesis is never expanded again; it stays in the history for the backtrace).
 *   states_in / states_out   HOST arrays of n_states DEVICE pointers, each [S*B, state_dim] fp32,
 *                            pitch state_dim; an array must not be its own output.
 *   backptr_dev, words_dev, scores_dev   device [max_len, S, B] (int32, int32, fp32), caller-owned.
 *   next_scores_dev          device fp32 [S*B]: the beam_scores of the next step; may be
 *                            out_score_dev itself (each entry is read before it is written).
 * Asynchronous on the stream, allocates nothing, one kernel. */
lsh_status lsh_beam_advance(const lsh_beam_params* bp, int32_t step, const int32_t* out_beam_dev,
                            const int32_t* out_word_dev, const float* out_score_dev,
                            const float* const* states_in, float* const* states_out,
                            int32_t* backptr_dev, int32_t* words_dev, float* scores_dev,
                            float* next_scores_dev, void* hip_stream);

/* After n_steps recorded steps: per sentence the best finished hypothesis (a slot whose word is
 * eos) over all steps -- highest score, then earliest step, then lowest slot -- or, if none
 * finished, the best slot of the last step; its words in order, found by walking the parent
 * pointers back to step 0.
 *   tokens_dev int32 [S, max_len] (only the first length[s] entries of a row are written),
 *   length_dev int32 [S] (0 if nothing was recorded), best_score_dev fp32 [S]. */
lsh_status lsh_beam_backtrace(const lsh_beam_params* bp, int32_t n_steps, const int32_t* backptr_dev,
                              const int32_t* words_dev, const float* scores_dev, int32_t* tokens_dev,
                              int32_t* length_dev, float* best_score_dev, void* hip_stream);

/* ---- inspection (synchronous device-to-host copies; never on the timed path) ---------------- */

/* Band codes (Eq. 6-8) of R fp32 rows of pitch d, computed by the same device hash routine the
 * step uses.  codes_host is int32 [R, W]. */
lsh_status lsh_debug_codes(const lsh_tables* t, const float* H_dev, int32_t R, int32_t* codes_host);

/* Band codes of the embedding rows [row0, row0+n) as computed at build time; int32 [n, W]. */
lsh_status lsh_debug_embedding_codes(const lsh_tables* t, int32_t row0, int32_t n,
                                     int32_t* codes_host);

/* T_w[code] read THROUGH the device cuckoo table: *n_out = span length or -1 if the code has no
 * bucket; up to cap ids are written. */
lsh_status lsh_debug_bucket(const lsh_tables* t, int32_t band, int32_t code, int32_t* words_host,
                            int32_t cap, int32_t* n_out);

/* The flat layout of one band: distinct codes ascending, span offsets, word ids [V]. */
lsh_status lsh_debug_csr(const lsh_tables* t, int32_t band, int32_t* n_keys_out, int32_t* keys_host,
                         int32_t* offsets_host, int32_t cap_keys, int32_t* words_host);

/* Slots in one band's cuckoo table and keys stored (capacity is a power of two >= 2 * keys). */
lsh_status lsh_debug_cuckoo_shape(const lsh_tables* t, int32_t band, int32_t* capacity_out,
                                  int32_t* n_keys_out);

/* How the tables were built: *on_device_out = 1 if sort and cuckoo insertion ran on the device
 * (0: on the host, after the device insertion had given up or by request); *attempts_out =
 * insertion rounds the device made (bands whose insertion fails are redone with new hash
 * parameters). */
lsh_status lsh_debug_build_info(const lsh_tables* t, int32_t* on_device_out, int32_t* attempts_out);

/* Candidate list of sentence s left in the workspace by the last LSH step on it. */
lsh_status lsh_debug_candidates(const lsh_tables* t, const void* workspace_dev,
                                const lsh_step_params* sp, int32_t s, int32_t* cand_host,
                                int32_t cap, int32_t* n_out);

/* Candidate counts |V_LSH,s| of all S sentences from the last step on this workspace (V for a
 * full-vocabulary step); counts_host is int32 [S]. */
lsh_status lsh_debug_counts(const lsh_tables* t, const void* workspace_dev, const lsh_step_params* sp,
                            int32_t* counts_host);

/* Log-probabilities of sentence s from the last step on this workspace: lp_host is fp32
 * [B, cap] (row pitch cap), columns in candidate-list order; *n_out = candidate count. */
lsh_status lsh_debug_logprobs(const lsh_tables* t, const void* workspace_dev,
                              const lsh_step_params* sp, int32_t s, float* lp_host, int32_t cap,
                              int32_t* n_out);

/* ---- launch-plan options (for tests and measurements; no effect on results) -------------------
 *
 * A step chooses its kernels from the shape (few sentences: one fused kernel; many: separate
 * candidate, contraction and selection kernels; ...).  Every rule can be overridden per handle.
 * `value` >= 0 forces, LSH_OPTION_AUTO restores the library's rule.  When a handle is built, each
 * option takes the value of the environment variable LSHBEAM_<NAME IN CAPITALS> if that is set
 * (read once, inside lsh_build_tables); lsh_decode_step never reads the environment.  Not
 * synchronised with steps running on the handle from other threads: set options between steps.
 *   "fused"          1 / 0: candidate generation inside the contraction kernel, or separate kernels
 *   "one_launch"     0: the fused kernel is followed by a selection kernel instead of running the
 *                    selection in its last workgroup
 *   "fused_grid"     workgroups of the fused kernel (default 256)
 *   "fused_tile"     n = 1..15: candidates per tile of the fused kernel instead of 16
 *   "logits_grid"    workgroups (or waves' worth of them) of the separate contraction kernels
 *   "logits_waves"   1 / 4 / 16: contraction driver (a wave per tile; k split over 4 or 16 waves)
 *   "logits_hlds"    0: the wave-per-tile driver keeps the hidden rows in global memory, not LDS
 *   "logits_estage"  0: 33..64 beams take the grouped driver instead of candidate rows through LDS
 *   "estage_union"   0: sentences hashed in parts get their candidate list from a kernel of its own
 *                    before that driver, instead of inside it
 *   "hlds_rem"       n: a last round of tiles filling at most 1/n of the waves is split over k (4)
 *   "logits_planes"  0: bf16 rows are widened to fp32 instead of meeting bf16 planes of H
 *   "hlds_rows"      16 / 32: hidden rows per group of the LDS-staged driver
 *   "part_rows"      n: sentences are hashed in parts of n rows, a workgroup each
 *   "stage_rows"     n: the hashing stage in LDS is sized for at most n rows (0: the minimum)
 * Two more are read from the environment by lsh_build_tables only: LSHBEAM_HOST_BUILD=1 (bucket and
 * cuckoo tables built on the host) and LSHBEAM_CUCKOO_CHAIN=n (eviction chains of the device
 * build cut at n; for tests of its retry path). */
#define LSH_OPTION_AUTO (-1)
lsh_status lsh_set_option(lsh_tables* t, const char* name, int32_t value);
lsh_status lsh_get_option(const lsh_tables* t, const char* name, int32_t* value_out);

/* ---- per-kernel timing -------------------------------------------------------------------- */

#define LSH_NUM_KERNELS 5 /* 0 candidates (hash+probe+merge, or union of earlier bitmaps +
                             compaction), 1 gathered logits, 2 select, 3 per-row hit counts
                             (t > 1 only), 4 per-part hashing (sentences with many beams) */

/* 1 if a step with these parameters runs candidate generation inside the logits kernel (steps
 * with little work: few sentences; the timing slot 0 then stays empty and slot 1 covers the
 * fused kernel `k_cand_logits`, or `k_union_logits` when slots 3 or 4 ran first), 0 if it runs
 * the kernels separately. */
int32_t lsh_step_is_fused(const lsh_tables* t, const lsh_step_params* sp);

/* A profiler owns device start/stop events for up to max_launches launches of each kernel.  The
 * caller owns it and hands it to the steps it wants timed; the tables handle holds no timing
 * state, so steps on different streams can be timed with different profilers.  One profiler must
 * not be used by two steps at the same time. */
typedef struct lsh_profiler lsh_profiler;
lsh_status lsh_profiler_create(int32_t max_launches, lsh_profiler** out);
void lsh_profiler_destroy(lsh_profiler* p); /* NULL-safe */

/* lsh_decode_step with the device start/stop time of each of its kernel launches recorded in
 * `prof` (NULL: exactly lsh_decode_step).  Launches beyond max_launches are not recorded. */
lsh_status lsh_decode_step_timed(const lsh_tables* t, const float* H_dev, const float* beam_scores_dev,
                                 const int32_t* topfreq_dev, const lsh_step_params* sp,
                                 void* workspace_dev, size_t workspace_bytes, int32_t* out_beam_dev,
                                 int32_t* out_word_dev, float* out_score_dev, void* hip_stream,
                                 lsh_profiler* prof);

/* Synchronises the device, writes the mean duration in milliseconds per launch of each kernel and
 * the number of recorded launches, and empties the profiler for reuse.  A step launches each
 * kernel at most once; callers that compute time per step as mean x launches / steps stay correct
 * should that change. */
lsh_status lsh_profiler_read(lsh_profiler* p, double mean_ms_out[LSH_NUM_KERNELS],
                             int32_t launches_out[LSH_NUM_KERNELS]);
const char* lsh_kernel_name(int32_t which);

const char* lsh_status_string(lsh_status s);

#ifdef __cplusplus
}
#endif
#endif /* LSHBEAM_H */
