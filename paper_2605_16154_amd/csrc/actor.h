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

struct ActorIO {
    const void* hidden;
    const uint8_t* tokens;
    const float* logp_old;
    const float* adv;
    const int32_t* kept_idx;
    const int32_t* n_kept;
    const void *Wg, *Wu, *Wd, *Wo;
    float eps_low, eps_high, loss_scale;
    float* loss_out;
    float* logp_out;
    float *dWg, *dWu, *dWd, *dWo;
    void* dX;
    float* stats_out;
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
};

// gather.hip ---------------------------------------------------------------------------------
// Copies the kept chunks' hidden rows into X [rows_pad, d] (rows at and beyond n_kept*A are
// zero-filled) and fills the row metadata.  elem_bytes is 2 (bf16) or 4 (fp32).
int launch_gather(const ActorShape& sh, const ActorIO& io, int elem_bytes, void* X, int64_t rows_pad,
                  RowMeta meta, hipStream_t s);

// Sums the per-row loss terms and statistics in a fixed order (one workgroup, fp64 accumulators).
int launch_loss_reduce(const ActorShape& sh, const ActorIO& io, RowOut out, hipStream_t s);

// Row-wise loss math shared by both paths (device).  Returns the coefficient c such that
// dz = c * (onehot - softmax): c = -loss_scale * rho * A when the gradient flows, else 0.
struct LossRow {
    float term, ratio, dlogp, coef;
    uint8_t clipped;
};
__device__ inline LossRow loss_row(float logp, float logp_old, float adv, float eps_low, float eps_high,
                                   float loss_scale) {
    LossRow r;
    r.dlogp = logp_old - logp;
    r.ratio = expf(logp - logp_old);
    const float lo = 1.f - eps_low, hi = 1.f + eps_high;
    const float clipped_ratio = fminf(fmaxf(r.ratio, lo), hi);
    r.term = fminf(r.ratio * adv, clipped_ratio * adv);
    const bool flows = (adv >= 0.f && r.ratio <= hi) || (adv < 0.f && r.ratio >= lo);
    r.clipped = flows ? 0 : 1;
    r.coef = flows ? -loss_scale * r.ratio * adv : 0.f;
    return r;
}

// actor_f32.hip / actor_bf16.hip ---------------------------------------------------------------
size_t actor_f32_workspace_bytes(const ActorShape& sh, bool want_grads);
int actor_f32_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s);
size_t actor_bf16_workspace_bytes(const ActorShape& sh, bool want_grads);
int actor_bf16_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s);

}  // namespace pcm
