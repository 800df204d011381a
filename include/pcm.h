/*
 * pcm.h -- C boundary of the MI355X (gfx950) library for Probabilistic Chunk Masking (PCM)
 * and the masked GRPO actor step it feeds.
 *
 * One training step of the paper's Algorithm 1 maps onto four calls, in this order:
 *
 *   pcm_score_phases        advantages (Eq. 1) and the batch phase score C_c^(t) (Eq. 5)
 *   pcm_update_keep_probs   score buffers, share/max normalisation, keep probabilities (Eq. 7-9)
 *   pcm_sample_chunks       fixed-budget weighted sampling without replacement (Eq. 10) and
 *                           physical shrinking expressed as compacted chunk ids (Sec. 4.5)
 *   grpo_masked_actor_step  gather of the kept chunks, action-head forward, clipped GRPO
 *                           surrogate (Eq. 11; Eq. 2 when every chunk is kept) and backward
 *
 * and, to complete the actor update, pcm_adamw_clip_step applies the gradients (App. D).
 *
 * Conventions common to every entry point
 *   - Return value: PCM_OK or a negative pcm_status.  Nothing throws, aborts or prints.
 *   - "device" pointers are HIP device memory owned by the caller; they must stay valid until
 *     `stream` has executed the call.  "host" values are plain arguments.  The library never
 *     allocates or frees device memory and never synchronises the stream or the device: all
 *     work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Scratch memory comes from the caller: `workspace` (device, 256-byte aligned) of at least
 *     the size returned by the matching *_workspace_bytes query (host-only, no GPU work).  Its
 *     contents on entry are irrelevant; two calls that share a workspace must be ordered on
 *     one stream.
 *   - Argument checks are made on host scalars and on pointer nullness only; device data is
 *     never read by the host.  Out-of-range device data is never dereferenced out of bounds: a
 *     phase id >= K counts as phase K-1 in every call, a token >= V as V-1, n_chunks is clamped
 *     to [0, N], a chunk id outside [0, T*N) is treated as stated per call.
 *   - Layouts are dense row-major; T = n_groups * G trajectories, the G rollouts of group g
 *     being rows g*G .. g*G+G-1; N chunk slots per trajectory; A = L*D action values (and
 *     action tokens) per chunk (8 * 7 = 56 in the paper's setup, Sec. 5.1).
 */
#ifndef PCM_H_
#define PCM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PCM_OK = 0,
    PCM_EINVAL = -1,       /* null pointer, non-positive size, value out of the stated range */
    PCM_EWORKSPACE = -2,   /* workspace missing, misaligned or smaller than the query says */
    PCM_EHIP = -3,         /* a HIP call (kernel launch, event) reported an error */
    PCM_EUNSUPPORTED = -4  /* shape or dtype outside what the kernels implement */
} pcm_status;

typedef enum { PCM_F32 = 0, PCM_BF16 = 1 } pcm_dtype;

/* Exported symbols (the library is built with hidden default visibility). */
#if defined(__GNUC__)
#define PCM_API __attribute__((visibility("default")))
#else
#define PCM_API
#endif

/* Limits of the kernels (host-checked). */
#define PCM_MAX_PHASES 64        /* K */
#define PCM_MAX_CHUNK_SLOTS 4096 /* N */
#define PCM_MAX_OPT_TENSORS 8    /* tensors per optimizer call */

/* Library version string (host). */
PCM_API const char* pcm_version(void);
/* Short text for a status code (host). */
PCM_API const char* pcm_status_string(int status);

/* ------------------------------------------------------------------------------------------
 * Keep-probability state (Eq. 7-9; Algorithm 1: buffer initialisation, append, refresh).
 *
 * A flat block in device memory, trivially copyable (it is the only state PCM carries between
 * steps, so copying it out and back is a checkpoint).  Layout, all 8-byte words:
 *   int64 step; int64 since_refresh; double S[K]; int64 count[K]; double p[K]
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t pcm_state_bytes(int K);
/* device state: step = 0, buffers empty, p_c = 1.  Enqueued on stream. */
PCM_API int pcm_state_init(void* state, int K, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_label_phases -- the deterministic gripper-based phase label of every chunk (App. D, phase
 * allotment rules); produces the `phase` input of pcm_score_phases and pcm_sample_chunks.
 *
 * A timestep's gripper-close command is active when actions[.., t*D + gripper_dim] exceeds
 * close_threshold; g_f of a chunk is the fraction of its L timesteps with an active command.
 * Chunks with g_f >= 0.75 are "sustained close"; maximal runs of them are the grasp intervals.
 * Labels, highest priority first:
 *   2 active-grip    g_f >= 0.5
 *   1 pre-grasp      one of the three chunks right before a grasp interval and 0.1 <= g_f < 0.5
 *   3 release-ramp   one of the three chunks right after a grasp interval (g_f < 0.5)
 *   0 approach       g_f < 0.5 and a grasp interval begins later in the trajectory, or the
 *                    trajectory has no grasp interval at all
 *   4 tail           the rest: after the last grasp interval and outside its release window
 * (so K = 5).  The outcome of the rollout is not an input.
 *
 *   actions   device f32 [T, N, L*D]: per chunk, L timesteps of D values
 *   n_chunks  device i32 [T] or NULL (all N); clamped to [0, N]; slots beyond it get label 0
 *   phase     device u8 [T, N], written
 * Errors: PCM_EINVAL for null pointers, N > PCM_MAX_CHUNK_SLOTS, gripper_dim outside [0, D),
 * NaN threshold, non-positive sizes.
 * ------------------------------------------------------------------------------------------ */
PCM_API int pcm_label_phases(const float* actions, const int32_t* n_chunks, int T, int N, int L, int D,
                     int gripper_dim, float close_threshold, uint8_t* phase, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_score_phases -- Eq. 1 and Eq. 5 (with the skip rule of App. D.2, last paragraph).
 *
 * For every group with both outcomes and every phase c: pool the group's chunks of phase c
 * (chunk slot k < n_chunks[i]) into successes (reward 1) and failures (reward 0); the pair's
 * score is the Euclidean norm of the difference of the two pooled mean action vectors; a pair
 * missing either outcome is skipped.  C_out[c] is the mean of the pair scores over the groups
 * that were not skipped, valid_out[c] whether any group contributed (C_out[c] = 0 if none).
 * Groups whose rewards are all equal are ignored for the score and get advantage 0, active 0.
 *
 * Exactness: actions enter as integers rint(a * 2^24); sums are 64-bit integers, so the result
 * does not depend on launch geometry or summation order; the remaining fp64 operations are
 * done in a fixed order without fused multiply-add.  Required: |a| <= 2^20, finite.
 *
 *   actions   device f32 [T, N, A]
 *   phase     device u8  [T, N]; entries >= K count as phase K-1 (the same rule as in pcm_sample_chunks)
 *   reward    device u8  [T]; non-zero = success
 *   n_chunks  device i32 [T] valid chunk slots per trajectory (clamped to [0, N]); NULL = all N
 *   adv_eps   host, epsilon of Eq. 1 (>= 0)
 *   C_out     device f64 [K];  valid_out device u8 [K]
 *   adv_out   device f32 [T] or NULL;  active_out device u8 [T] or NULL
 * Limits: 1 <= K <= PCM_MAX_PHASES, 1 <= A <= 256, G >= 1, n_groups >= 1, N >= 1.
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t pcm_score_phases_workspace_bytes(int n_groups, int G, int N, int A, int K);
PCM_API int pcm_score_phases(const float* actions, const uint8_t* phase, const uint8_t* reward,
                     const int32_t* n_chunks, int n_groups, int G, int N, int A, int K,
                     double adv_eps, double* C_out, uint8_t* valid_out, float* adv_out,
                     uint8_t* active_out, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_score_phases_static -- pcm_score_phases for callers that cannot provide or allocate a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without the workspace pair), same kernels, same results; the
 * accumulators live in a fixed array of PCM_SCORE_STATIC_MAX_BYTES bytes inside the library, of
 * which every GPU the library runs on holds one copy until the process ends.  The call allocates
 * and frees nothing (its first call on a device looks up that device's copy of the array).
 *
 * Errors: as pcm_score_phases; PCM_EWORKSPACE when pcm_score_phases_workspace_bytes(...) of the
 * shape exceeds PCM_SCORE_STATIC_MAX_BYTES (about n_groups * K * A * 16 bytes: the paper-sized
 * batch needs 0.07 MB, 64 groups of 12 phases 0.7 MB).
 * All calls on one GPU share that GPU's array: two calls that may overlap (different streams
 * without an ordering between them, or different host threads) race; order them.
 * ------------------------------------------------------------------------------------------ */
#define PCM_SCORE_STATIC_MAX_BYTES (4u << 20)   /* 4 MiB */
PCM_API int pcm_score_phases_static(const float* actions, const uint8_t* phase, const uint8_t* reward,
                     const int32_t* n_chunks, int n_groups, int G, int N, int A, int K,
                     double adv_eps, double* C_out, uint8_t* valid_out, float* adv_out,
                     uint8_t* active_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_update_keep_probs -- Eq. 7 (append), Eq. 8 (collapse), Eq. 9 (floor); Sec. 4.3-4.4.
 *
 * Appends the valid scores to the per-phase buffers (kept as running sums).  On the first call
 * after pcm_state_init and then whenever T_rc calls have been appended since the last refresh:
 * rho~_c = S_c / max_c' S_c' (0 if every S is 0), p_c = max(p_min, rho~_c), buffers reset.
 * Otherwise p is left as it was.  keep_probs_out receives a copy of p either way.
 *
 *   state  device block of pcm_state_bytes(K);  C device f64 [K];  valid device u8 [K]
 *   p_min  host, in (0, 1];  T_rc host, >= 1;  keep_probs_out device f64 [K] or NULL
 * ------------------------------------------------------------------------------------------ */
PCM_API int pcm_update_keep_probs(void* state, const double* C, const uint8_t* valid, int K, double p_min,
                          int T_rc, double* keep_probs_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_sample_chunks -- Eq. 10 and the shrinking step of Algorithm 1's inner loop (Sec. 4.5).
 *
 * Every chunk slot k < n_chunks[i] of an active trajectory i carries the integer weight
 * q = clamp(floor(p_phase * 2^16 + 0.5), 1, 2^16) of its phase (phase ids >= K use phase K-1).
 * min(B, n_chunks[i]) chunks are drawn by successive weighted sampling without replacement:
 * round r takes 64 random bits x = Philox4x32-10(counter = (i, r, step low, step high),
 * key = (seed low, seed high)), words 0 and 1, maps them to t = floor(x * W_rem / 2^64) and
 * picks the first remaining slot whose inclusive running weight exceeds t.  The draw depends
 * only on (seed, step, i, r), not on launch geometry.  Inactive trajectories keep nothing.
 *
 *   keep_probs device f64 [K];  phase device u8 [T, N];  n_chunks device i32 [T] or NULL
 *   active     device u8 [T] or NULL (= all active)
 *   kept_idx     device i32 [T * min(B, N)]: global chunk ids i*N + k, ascending; entries at
 *                and beyond *n_kept are left untouched
 *   kept_offsets device i32 [T + 1]: exclusive scan of per-trajectory kept counts
 *   n_kept       device i32 [1] = kept_offsets[T]
 * Limits: 1 <= K <= PCM_MAX_PHASES, 1 <= N <= PCM_MAX_CHUNK_SLOTS, B >= 1, T >= 1,
 *         T * N < 2^31.
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t pcm_sample_chunks_workspace_bytes(int T, int N, int K, int B);
PCM_API int pcm_sample_chunks(const double* keep_probs, const uint8_t* phase, const int32_t* n_chunks,
                      const uint8_t* active, int T, int N, int K, int B, uint64_t seed,
                      uint64_t step, int32_t* kept_idx, int32_t* kept_offsets, int32_t* n_kept,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_sample_chunks_ex -- pcm_sample_chunks with a choice of selector: the method, or one of the
 * two ablations that bracket it (Sec. 5.2, RQ4).  All other arguments as pcm_sample_chunks.
 *   PCM_SELECT_PCM        weights = the phases' keep probabilities (the method, Eq. 10)
 *   PCM_SELECT_RANDOM     equal weights: min(B, N_i) chunks uniformly at random; keep_probs is
 *                         not used for the weights (it must still point at K doubles)
 *   PCM_SELECT_TOP_PHASE  only chunks of the one phase with the largest keep probability (lowest
 *                         index on ties) are eligible, with equal weights; a trajectory keeps
 *                         min(B, its chunks in that phase), possibly none
 *   PCM_SELECT_STRATIFIED the scheme the variance analysis of App. C assumes (Theorem 1): a fixed
 *                         budget b_c per phase, then b_c chunks of phase c uniformly without
 *                         replacement.  With q_c = clamp(floor(p_c 2^16 + 0.5), 1, 2^16), N_c the
 *                         trajectory's valid chunks in phase c, m = min(B, N_i), D = sum N_c q_c:
 *                         b_c = min(N_c, floor(m N_c q_c / D)); the chunks left over go one at a
 *                         time to the phase with the largest (m N_c q_c) mod D that still has
 *                         room (lowest index on ties), round after round.  Draws run through the
 *                         phases in index order with one draw counter.
 *
 * pcm_importance_weights -- the weights N_c / b_c of the ratio estimator (App. C, the unbiased
 * alternative to Eq. 11), one per kept chunk, for grpo_masked_actor_step_ex's chunk_weight:
 * N_c = valid chunks of the kept chunk's phase in its trajectory, b_c = kept ones among them.
 *   kept_idx, kept_offsets  device, as written by pcm_sample_chunks
 *   weights   device f32 [kept_offsets[T]]: entry j belongs to kept_idx[j]
 * ------------------------------------------------------------------------------------------ */
typedef enum {
    PCM_SELECT_PCM = 0,
    PCM_SELECT_RANDOM = 1,
    PCM_SELECT_TOP_PHASE = 2,
    PCM_SELECT_STRATIFIED = 3
} pcm_selector;
PCM_API int pcm_sample_chunks_ex(const double* keep_probs, const uint8_t* phase, const int32_t* n_chunks,
                         const uint8_t* active, int T, int N, int K, int B, int selector,
                         uint64_t seed, uint64_t step, int32_t* kept_idx, int32_t* kept_offsets,
                         int32_t* n_kept, void* workspace, size_t workspace_bytes, void* stream);
PCM_API int pcm_importance_weights(const uint8_t* phase, const int32_t* n_chunks, const int32_t* kept_idx,
                           const int32_t* kept_offsets, int T, int N, int K, float* weights,
                           void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_kept_phase_counts -- the realised allocation of the budget over the phases (Sec. 5.2, the
 * per-phase view of which chunks were kept): a statistic for logging, not a step of the update.
 *
 *   phase, n_chunks, active   device, as given to pcm_sample_chunks (n_chunks, active may be NULL)
 *   kept_idx, n_kept          device, as written by pcm_sample_chunks; *n_kept is clamped to
 *                             [0, max_kept_chunks], ids outside [0, T*N) are not counted
 *   kept_per_phase    device i32 [K]: kept chunks of each phase (ids >= K count as K-1)
 *   chunks_per_phase  device i32 [K] or NULL: chunk slots the sampler could have kept (slots
 *                     k < n_chunks[i] of active trajectories) of each phase
 * One workgroup; meant for batches of up to a few million chunk slots.
 * ------------------------------------------------------------------------------------------ */
PCM_API int pcm_kept_phase_counts(const uint8_t* phase, const int32_t* n_chunks, const uint8_t* active,
                          const int32_t* kept_idx, const int32_t* n_kept, int max_kept_chunks, int T, int N,
                          int K, int32_t* kept_per_phase, int32_t* chunks_per_phase, void* stream);

/* ------------------------------------------------------------------------------------------
 * grpo_masked_actor_step -- Eq. 11 (Eq. 2 when kept_idx lists every chunk), with the PPO
 * clipping the paper leaves out of Eq. 2 for clarity (thresholds as in App. D).
 *
 * Rows are the A action tokens of each kept chunk, in kept order: row r of the compacted batch
 * is token r % A of chunk kept_idx[r / A], i.e. row kept_idx[r / A] * A + r % A of `hidden`.
 * Head (weights stored [in, out], no bias): u = x Wg, v = x Wu, a = silu(u) * v, y = a Wd,
 * z = y Wo (V logits).  Per row: l = log softmax(z)[token], rho = exp(l - logp_old),
 * term = min(rho * A_i, clip(rho, 1 - eps_low, 1 + eps_high) * A_i) with A_i the advantage of
 * the chunk's trajectory; loss = -loss_scale * sum of terms over the first *n_kept chunks.
 * Gradients are those of that loss; a ratio exactly on a clip boundary counts as unclipped.
 *
 *   hidden    device [T*N*A, d] of dtype;  tokens device u8 [T*N*A] (values >= V use V-1)
 *   logp_old  device f32 [T*N*A];  adv device f32 [T]
 *   kept_idx  device i32 [>= max_kept_chunks]; ids outside [0, T*N) are treated as id 0 with
 *             advantage 0;  n_kept device i32 [1], clamped to [0, max_kept_chunks]
 *   Wg, Wu    device [d, ff];  Wd device [ff, d];  Wo device [d, V]  (dtype)
 *   loss_out  device f32 [1]
 *   logp_out  device f32 [max_kept_chunks * A] or NULL (rows beyond the kept ones: untouched)
 *   dWg, dWu  device f32 [d, ff]; dWd device f32 [ff, d]; dWo device f32 [d, V]: overwritten.
 *             Pass all four NULL (and dX NULL) for a forward-only call.
 *   dX        device [max_kept_chunks * A, d] of dtype, or NULL
 *   stats_out device f32 [4] or NULL: fraction of rows with clipped (zero) gradient, mean rho,
 *             mean (logp_old - l), number of rows
 * dtype PCM_F32: fp32 storage and arithmetic; any d, ff >= 1, 1 <= V <= 1024.
 * dtype PCM_BF16: bf16 storage, MFMA with fp32 accumulation, bf16 intermediates;
 *             requires d % 256 == 0, ff % 256 == 0, V == 256.
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t grpo_masked_actor_step_workspace_bytes(int max_kept_chunks, int A, int d, int ff, int V,
                                              int dtype, int want_grads);
PCM_API int grpo_masked_actor_step(const void* hidden, const uint8_t* tokens, const float* logp_old,
                           const float* adv, const int32_t* kept_idx, const int32_t* n_kept,
                           int max_kept_chunks, int T, int N, int A, int d, int ff, int V,
                           int dtype, const void* Wg, const void* Wu, const void* Wd,
                           const void* Wo, float eps_low, float eps_high, float loss_scale,
                           float* loss_out, float* logp_out, float* dWg, float* dWu, float* dWd,
                           float* dWo, void* dX, float* stats_out, void* workspace,
                           size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * grpo_masked_actor_step_ex -- the same step with the variants of the training loss (App. D,
 * training details: asymmetric clipping (0.2, 0.4), entropy coefficient 1e-3; App. C: the
 * importance-weighted unbiased estimator).  All other arguments as grpo_masked_actor_step.
 *
 * With M = (*n_kept) * A live rows, scale = loss_scale (PCM_NORM_SCALE) or loss_scale / M
 * (PCM_NORM_TOKEN_MEAN; 0 when M = 0), w_c = chunk_weight[c] for the c-th kept chunk (1 if NULL),
 * H_r the entropy of row r's distribution over the V bins:
 *   PCM_RATIO_TOKEN  rho_r = exp(l_r - logp_old_r);   T = sum over rows of w_c min(rho_r A_i, clip(rho_r) A_i)
 *   PCM_RATIO_CHUNK  rho_c = exp(sum over the chunk's A rows of (l_r - logp_old_r)), the ratio of
 *                    the chunk's probabilities (Eq. 2 is written per chunk);
 *                    T = sum over chunks of w_c min(rho_c A_i, clip(rho_c) A_i)
 *   loss = -scale * T - entropy_coef * scale * sum over rows of H_r
 * Gradients are those of that loss.
 *
 * head_evaluation chooses how the two linear maps after the gated activation a are applied:
 *   PCM_HEAD_AS_WRITTEN  y = a Wd, z = y Wo, and in the backward pass dWo = y^T dz, dy = dz Wo^T,
 *                        dWd = a^T dy, da = dy Wd^T;
 *   PCM_HEAD_COMPOSED    as one matrix W_do = Wd Wo [ff, V], formed inside the call from the
 *                        current weights: z = a W_do; G = a^T dz, dWd = G Wo^T, dWo = Wd^T G,
 *                        da = dz W_do^T.  The same function and the same gradients in exact
 *                        arithmetic (only a linear map sits between the two projections); with
 *                        V much smaller than d the three large products through d (down, dWd, da)
 *                        become products through the V-wide bottleneck, about 30 % fewer
 *                        multiply-adds for the whole step.  Rounding differs: y and dy are
 *                        never formed (nor rounded to bf16), W_do and G are rounded instead.
 *
 *   options    host pointer, read during the call only
 *   options->chunk_weight  device f32 [max_kept_chunks] or NULL (e.g. N_c / b_c: chunks of the
 *              chunk's phase in its trajectory over those kept)
 *   stats_out  device f32 [5] or NULL: as grpo_masked_actor_step (with a per-chunk ratio, entries 0
 *              and 1 use the chunk's ratio for each of its rows), then the mean row entropy
 * Row panels (dtype PCM_BF16, PCM_HEAD_AS_WRITTEN; grpo_masked_actor_step does the same with the default
 * height): a batch longer than a panel and a quarter is worked through in panels of the largest common multiple
 * of 256 and A that does not exceed the target height: gather, forward, loss and backward run panel by panel
 * over the same activation buffers, every panel after the first adds its weight gradients to the earlier ones'
 * (fp32), the loss is reduced once at the end.  The workspace is bounded by the panel, not by the batch.
 *
 * Rows without a gradient (dtype PCM_BF16, PCM_HEAD_AS_WRITTEN, entropy_coef == 0; grpo_masked_actor_step does the
 * same): a row whose ratio the clip cuts, or whose advantage or chunk weight is zero, has an all-zero row of
 * d loss / d logits (Eq. 11 with the clipped surrogate), so it adds nothing to any weight gradient and its row of dX
 * is zero.  When at least one row in sixteen of a panel is such a row, the backward products run over the other rows
 * only (copied into dense operands; the decision is taken on the device from the loss stage's results).  The
 * outputs are those of the backward pass over all rows up to the order of the fp32 sums.  dense_backward != 0
 * switches this off.
 *
 * Precision of PCM_RATIO_CHUNK with dtype PCM_BF16: the log-probabilities of a chunk's A rows add up in the
 * exponent of its ratio, and so would their bf16 errors (about 2e-3 each, 2e-2 for A = 56).  The forward pass
 * therefore carries a and y as pairs of bf16 values (value + rounding remainder) through the down and the logit
 * product (twice the multiply-adds of those two products; workspace for the two remainders), which keeps the
 * gradients within the 2e-2 bound of the per-token form at any A.  That pass exists for PCM_HEAD_AS_WRITTEN only:
 * PCM_RATIO_CHUNK with PCM_HEAD_COMPOSED and PCM_BF16 returns PCM_EUNSUPPORTED.
 * Errors: PCM_EINVAL also for options == NULL, an unknown normalisation, ratio_level or
 * head_evaluation, NaN coefficients, negative panel_rows, misaligned packed_weights; PCM_EUNSUPPORTED for
 * packed_weights with dtype PCM_F32 or PCM_HEAD_COMPOSED.
 * ------------------------------------------------------------------------------------------ */
typedef enum { PCM_NORM_SCALE = 0, PCM_NORM_TOKEN_MEAN = 1 } pcm_normalisation;
typedef enum { PCM_RATIO_TOKEN = 0, PCM_RATIO_CHUNK = 1 } pcm_ratio_level;
typedef enum { PCM_HEAD_AS_WRITTEN = 0, PCM_HEAD_COMPOSED = 1 } pcm_head_evaluation;
typedef struct {
    float eps_low, eps_high;    /* clip thresholds (App. D: 0.2, 0.4) */
    float loss_scale;
    float entropy_coef;         /* App. D: 1e-3; 0 disables */
    int normalisation;          /* pcm_normalisation */
    int ratio_level;            /* pcm_ratio_level */
    const float* chunk_weight;  /* device, or NULL */
    int head_evaluation;        /* pcm_head_evaluation */
    int panel_rows;             /* dtype PCM_BF16: target height of the row panels a long batch is worked through in;
                                   0 = the library's choice (57,344 rows).  See "Row panels" above. */
    const void* packed_weights; /* device, or NULL: the operand layouts of the four weight matrices as written by
                                   pcm_pack_head_weights for these d, ff, V (dtype PCM_BF16, PCM_HEAD_AS_WRITTEN
                                   only).  The step then skips its own re-layout of Wg, Wu, Wd, Wo, which otherwise
                                   runs in every call although the weights change once per optimizer step.  The
                                   caller re-packs after every change of the weights; Wg, Wu, Wd, Wo must still be
                                   given (the backward pass reads them as they are). */
    int dense_backward;         /* dtype PCM_BF16: non-zero = backward products over all kept rows, also over rows
                                   without a gradient (see "Rows without a gradient" above); 0 = the default */
    double* grad_sumsq_out;     /* device f64 [1], 8-byte aligned, or NULL: receives the sum of the squares of all
                                   elements of dWg, dWu, dWd, dWo, gathered where their final values are written
                                   (fp64 throughout, summed in a fixed order), so that
                                   pcm_adamw_clip_step_ex needs no pass of its own over the gradients for the norm.
                                   dtype PCM_BF16, PCM_HEAD_AS_WRITTEN and all four gradients asked for; otherwise
                                   PCM_EUNSUPPORTED (PCM_EINVAL if misaligned). */
} pcm_loss_options;

/* ------------------------------------------------------------------------------------------
 * pcm_pack_head_weights -- the bf16 operand layouts that the forward products of the head read: gate and up
 * projection transposed and interleaved in blocks of 64 output columns ([2 ff, d], so that the gated activation
 * can be fused into the product), down projection transposed ([d, ff]), logit projection transposed ([V, d]).
 * The actor step builds them in its workspace on every call; a caller that keeps them (one pack per optimizer
 * step, after pcm_adamw_clip_step has written the bf16 weights) passes them in pcm_loss_options.packed_weights.
 *
 *   Wg, Wu device bf16 [d, ff];  Wd device bf16 [ff, d];  Wo device bf16 [d, V]
 *   packed  device, 256-byte aligned, pcm_packed_head_bytes(d, ff, V) bytes (0 = unsupported shape)
 * Requires d % 256 == 0, ff % 256 == 0, V == 256 (the shapes of the bf16 path).
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t pcm_packed_head_bytes(int d, int ff, int V);
PCM_API int pcm_pack_head_weights(const void* Wg, const void* Wu, const void* Wd, const void* Wo, int d, int ff, int V,
                          void* packed, void* stream);

/* Workspace of grpo_masked_actor_step_ex for these options (the per-chunk ratio needs more than the plain step). */
PCM_API size_t grpo_masked_actor_step_ex_workspace_bytes(int max_kept_chunks, int A, int d, int ff, int V, int dtype,
                                                 int want_grads, const pcm_loss_options* options);
PCM_API int grpo_masked_actor_step_ex(const void* hidden, const uint8_t* tokens, const float* logp_old,
                              const float* adv, const int32_t* kept_idx, const int32_t* n_kept,
                              int max_kept_chunks, int T, int N, int A, int d, int ff, int V,
                              int dtype, const void* Wg, const void* Wu, const void* Wd,
                              const void* Wo, const pcm_loss_options* options, float* loss_out,
                              float* logp_out, float* dWg, float* dWu, float* dWd, float* dWo,
                              void* dX, float* stats_out, void* workspace, size_t workspace_bytes,
                              void* stream);

/* ------------------------------------------------------------------------------------------
 * pcm_adamw_clip_step -- the optimizer step that follows the actor gradients (App. D, training
 * details: AdamW, constant learning rate 1e-5, betas (0.9, 0.999), weight decay 0, gradient
 * clipping at 2.0).
 *
 * With g the gradients of all n_tensors tensors taken together: norm = ||g||_2,
 * g <- g * min(1, max_grad_norm / (norm + 1e-6)); then per element, t = step (1 for the first
 * update):  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 * w <- w (1 - lr weight_decay) - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
 * The norm is accumulated in fp64 (in a fixed order: the result does not vary from run to run);
 * the update is fp32 arithmetic on fp32 state.
 *
 *   n_tensors     1 .. PCM_MAX_OPT_TENSORS
 *   numel         host i64 [n_tensors], each >= 1
 *   grads         host array of n_tensors device pointers, f32 [numel[i]]; read only
 *   weights, m, v host arrays of device pointers, f32 [numel[i]]; updated in place
 *   weights_bf16  NULL, or a host array of device pointers (entries may be NULL) to bf16
 *                 [numel[i]] that receive the new weights rounded to nearest even
 *   f32 pointers must be 16-byte aligned, bf16 pointers 8-byte aligned
 *   grad_norm_out device f32 [1] or NULL: the norm before clipping
 * Errors: PCM_EINVAL for a null or misaligned pointer or a hyper-parameter out of range (step < 1,
 * beta outside [0, 1), eps <= 0, negative lr / weight decay, max_grad_norm <= 0).
 *
 * pcm_adamw_clip_step_ex: the same with the sum of the squares of all gradient elements given (grad_sumsq, device
 * f64 [1], as grpo_masked_actor_step_ex leaves it in pcm_loss_options.grad_sumsq_out): the norm is its square root
 * and the gradients are read once, by the update.  grad_sumsq == NULL makes it pcm_adamw_clip_step.
 * ------------------------------------------------------------------------------------------ */
PCM_API size_t pcm_adamw_clip_step_workspace_bytes(int n_tensors, const int64_t* numel);
PCM_API int pcm_adamw_clip_step(int n_tensors, const int64_t* numel, const float* const* grads,
                                float* const* weights, float* const* m, float* const* v,
                                void* const* weights_bf16, int64_t step, double lr, double beta1,
                                double beta2, double eps, double weight_decay, double max_grad_norm,
                                float* grad_norm_out, void* workspace, size_t workspace_bytes,
                                void* stream);
PCM_API int pcm_adamw_clip_step_ex(int n_tensors, const int64_t* numel, const float* const* grads,
                                   float* const* weights, float* const* m, float* const* v,
                                   void* const* weights_bf16, int64_t step, double lr, double beta1,
                                   double beta2, double eps, double weight_decay, double max_grad_norm,
                                   const double* grad_sumsq, float* grad_norm_out, void* workspace,
                                   size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PCM_H_ */
