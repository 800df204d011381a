// Internal declarations for the masked GRPO actor step (Eq. 11): pieces shared by the fp32 and
// bf16 paths.  Not part of the C boundary.
#pragma once

#include <hip/hip_bf16.h>

#include "common.h"

namespace pcm {

using bf16 = __hip_bfloat16;

// Host scalars of one actor-step call.
struct ActorShape {
    int max_chunks;   // capacity of kept_idx (kept chunks at most)
    int T, N, A;      // trajectories, chunk slots per trajectory, tokens per chunk
    int d, ff, V;     // head sizes
    int64_t rows_max() const { return (int64_t)max_chunks * A; }
};

// How the objective is assembled from the rows (Eq. 11 plus the training details of App. D).
struct LossOptions {
    float eps_low, eps_high;     // clip thresholds
    float loss_scale;            // multiplies the summed objective
    float entropy_coef;          // subtracts entropy_coef * scale * sum of row entropies
    int token_mean;              // scale = loss_scale / (kept rows) instead of loss_scale
    int chunk_ratio;             // one ratio (and one clipped term) per chunk instead of per token
    const float* chunk_weight;   // device [max_chunks] or null: multiplies the terms of a chunk
    int panel_rows;              // bf16 path: target height of the row panels (0 = the library's choice)
    const void* packed_weights;  // bf16 path: operand layouts written by pcm_pack_head_weights, or null
    int dense_backward;          // bf16 path: backward products over all kept rows, also those without a gradient
    double* grad_sumsq_out;      // bf16 path: device [1] or null: sum of the squares of all four weight gradients
};

struct ActorIO {
    const void* hidden;
    const uint8_t* tokens;
    const float* logp_old;
    const float* adv;
    const int32_t* kept_idx;
    const int32_t* n_kept;
    const void *Wg, *Wu, *Wd, *Wo;
    LossOptions opt;
    float* loss_out;
    float* logp_out;
    float *dWg, *dWu, *dWd, *dWo;
    void* dX;
    float* stats_out;
    int n_stats;      // 4, or 5 when the mean row entropy is reported too
    bool composed;    // down and logit projection applied as one matrix Wd Wo (PCM_HEAD_COMPOSED)
    bool want_grads() const { return dWg != nullptr; }
};

// Per-row quantities produced by the gather and consumed by the loss stage.
struct RowMeta {
    uint8_t* token;    // [rows_pad] target bin (clamped to V-1)
    float* logp_old;   // [rows_pad]
    float* adv;        // [rows_pad] advantage of the row's trajectory; 0 for padding rows
};

// Per-row results of the loss stage, reduced in a fixed order afterwards.
struct RowOut {
    float* term;       // [rows_pad] min(rho A, clip(rho) A); 0 for padding rows
    float* ratio;      // [rows_pad]
    float* dlogp;      // [rows_pad] logp_old - logp
    uint8_t* clipped;  // [rows_pad] 1 if the row's gradient is cut by the clip
    float* entropy;    // [rows_pad] entropy of the row's distribution over the V bins
    float* coef;       // [rows_pad] per-chunk ratio only: factor of (onehot - softmax) in dz
};

// gather.hip ---------------------------------------------------------------------------------
// Copies the kept chunks' hidden rows into X [rows_pad, d] (rows at and beyond n_kept*A are
// zero-filled) and fills the row metadata.  elem_bytes is 2 (bf16) or 4 (fp32).
// With row_offset > 0 the rows are those of a panel of the batch that starts at that row: X and the metadata
// arrays are the panel's own, `rows_pad` its height.  The same holds for the two per-chunk-ratio launches below
// (row_offset a multiple of A, so no chunk straddles two panels).
int launch_gather(const ActorShape& sh, const ActorIO& io, int elem_bytes, void* X, int64_t row_offset, int64_t rows_pad,
                  RowMeta meta, hipStream_t s);

// Partial sums of squares of the four weight gradients, left by the launches that wrote their final values.
struct SumsqLists {
    const double* parts[4];
    int count[4];
};
// Sums the per-row loss terms and statistics in a fixed order (one workgroup, fp64 accumulators); with lists, also
// the partial sums of squares into io.opt.grad_sumsq_out.
int launch_loss_reduce(const ActorShape& sh, const ActorIO& io, RowOut out, const SumsqLists& lists, hipStream_t s);

// Per-chunk ratio: from the per-row dlogp, one ratio, one clipped term and one dz factor per kept chunk
// (written to every row of the chunk; the term only to its first row).
int launch_chunk_ratio(const ActorShape& sh, const ActorIO& io, RowMeta meta, RowOut out, int64_t row_offset,
                       int64_t rows_pad, hipStream_t s);

// dz[r, :] = coef[r] * dz[r, :] (+ extra[r, :] if extra is given) for the live rows r (V columns each);
// elem_bytes is 2 (bf16) or 4 (fp32).
int launch_scale_rows(const ActorShape& sh, const ActorIO& io, void* dz, const void* extra, const float* coef,
                      int64_t row_offset, int64_t rows_pad, int elem_bytes, hipStream_t s);

// Backward pass over the rows that carry a gradient only (bf16 path).  A kernel lists the panel's rows whose factor
// in dz is non-zero and writes, to device memory, what the backward products then read: their row count and which
// buffers hold their row-indexed operands (the panel's own, or copies of the listed rows).
struct LiveSources {
    static constexpr int kCount = 4;
    enum : int { kDz = 0, kY = 1, kA = 2, kX = 3 };
    const void* p[kCount];
};
struct LivePlan {
    const void* src[LiveSources::kCount];
    int32_t n_rows;    // rows of the backward products
    int32_t listed;    // 1: the products run over the listed rows (operands copied), 0: over all live rows
};
// A row carries a gradient when the clip does not cut it (RowOut::clipped) and its advantage and chunk weight are
// non-zero; clipped and adv are the panel's parts of those arrays.
int launch_live_row_list(const ActorShape& sh, const ActorIO& io, const uint8_t* clipped, const float* adv,
                         int64_t row_offset, int64_t rows_pad, const LiveSources& whole, const LiveSources& listed,
                         int32_t* idx, LivePlan* plan, hipStream_t s);
// dst[m] = src[idx[m]] (rows of row_bytes bytes, a multiple of 16) when the plan says listed; else nothing.
int launch_gather_listed(const void* src, const int32_t* idx, const LivePlan* plan, int64_t rows_pad, int64_t row_bytes,
                         void* dst, hipStream_t s);
// Zero rows of the panel's part of dX (rows_in_dX rows exist) wherever the listed products write nothing.
int launch_zero_unlisted(const ActorShape& sh, const ActorIO& io, const uint8_t* clipped, const float* adv,
                         int64_t row_offset, int64_t rows_pad, int64_t rows_in_dX, int64_t row_bytes, void* dX,
                         hipStream_t s);

// Number of live rows from the device-side kept count.
__device__ inline int64_t live_rows(const int32_t* n_kept, int max_chunks, int A) {
    int nk = *n_kept;
    nk = nk < 0 ? 0 : (nk > max_chunks ? max_chunks : nk);
    return (int64_t)nk * A;
}
// Factor in front of the summed objective.
__device__ inline float objective_scale(const LossOptions& o, int64_t rows_live) {
    if (!o.token_mean) return o.loss_scale;
    return rows_live > 0 ? o.loss_scale / (float)rows_live : 0.f;
}

// Clipped-surrogate math of one ratio (device), shared by both paths and both ratio levels.
// term = weight * min(rho A, clip(rho) A); coef is the factor c in dz = c * (onehot - softmax):
// c = -scale * weight * rho * A where the gradient flows, else 0.
struct LossRow {
    float term, ratio, dlogp, coef;
    uint8_t clipped;
};
__device__ inline LossRow loss_from_ratio(float ratio, float adv, float weight, const LossOptions& o, float scale) {
    LossRow r;
    r.dlogp = 0.f;
    r.ratio = ratio;
    const float lo = 1.f - o.eps_low, hi = 1.f + o.eps_high;
    const float clipped_ratio = fminf(fmaxf(ratio, lo), hi);
    r.term = weight * fminf(ratio * adv, clipped_ratio * adv);
    const bool flows = (adv >= 0.f && ratio <= hi) || (adv < 0.f && ratio >= lo);
    r.clipped = flows ? 0 : 1;
    r.coef = flows ? -scale * weight * ratio * adv : 0.f;
    return r;
}
__device__ inline LossRow loss_row(float logp, float logp_old, float adv, float weight, const LossOptions& o,
                                   float scale) {
    LossRow r = loss_from_ratio(expf(logp - logp_old), adv, weight, o, scale);
    r.dlogp = logp_old - logp;
    return r;
}

// actor_f32.hip / actor_bf16.hip ---------------------------------------------------------------
size_t actor_f32_workspace_bytes(const ActorShape& sh, bool want_grads);
int actor_f32_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s);
size_t actor_bf16_workspace_bytes(const ActorShape& sh, bool want_grads, const LossOptions& opt, bool composed);
int actor_bf16_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s);
size_t packed_head_bytes(int d, int ff, int V);
int pack_head_weights(const void* Wg, const void* Wu, const void* Wd, const void* Wo, int d, int ff, int V, void* packed,
                      hipStream_t s);

}  // namespace pcm
