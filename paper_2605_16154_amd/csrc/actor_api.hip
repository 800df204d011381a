// grpo_masked_actor_step: argument checks and dispatch to the fp32 or bf16 path.
#include "actor.h"

using namespace pcm;

namespace {

bool shape_supported(const ActorShape& sh, int dtype) {
    if (dtype == PCM_F32) return sh.V <= 1024;
    if (dtype == PCM_BF16) return sh.d % 256 == 0 && sh.ff % 256 == 0 && sh.V == 256;
    return false;
}

bool shape_valid(const ActorShape& sh) {
    return sh.max_chunks >= 1 && sh.A >= 1 && sh.d >= 1 && sh.ff >= 1 && sh.V >= 1 &&
           sh.rows_max() < ((int64_t)1 << 31) - 256;
}

}  // namespace

namespace {
size_t workspace_need(const ActorShape& sh, int dtype, bool bwd, const LossOptions& opt, bool composed) {
    return dtype == PCM_F32 ? actor_f32_workspace_bytes(sh, bwd) : actor_bf16_workspace_bytes(sh, bwd, opt, composed);
}
LossOptions plain_options(float eps_low, float eps_high, float loss_scale) {
    return LossOptions{eps_low, eps_high, loss_scale, 0.f, 0, 0, nullptr, 0, nullptr, 0, nullptr};
}
LossOptions from_boundary(const pcm_loss_options& o) {
    return LossOptions{o.eps_low, o.eps_high, o.loss_scale, o.entropy_coef, o.normalisation == PCM_NORM_TOKEN_MEAN,
                       o.ratio_level == PCM_RATIO_CHUNK, o.chunk_weight, o.panel_rows, o.packed_weights,
                       o.dense_backward != 0, o.grad_sumsq_out};
}
}  // namespace

extern "C" size_t grpo_masked_actor_step_workspace_bytes(int max_kept_chunks, int A, int d, int ff, int V,
                                                         int dtype, int want_grads) {
    ActorShape sh{max_kept_chunks, 1, 1, A, d, ff, V};
    if (!shape_valid(sh) || !shape_supported(sh, dtype)) return 0;
    return workspace_need(sh, dtype, want_grads != 0, plain_options(0.f, 0.f, 1.f), false);
}

extern "C" size_t grpo_masked_actor_step_ex_workspace_bytes(int max_kept_chunks, int A, int d, int ff, int V, int dtype,
                                                            int want_grads, const pcm_loss_options* options) {
    ActorShape sh{max_kept_chunks, 1, 1, A, d, ff, V};
    if (!options || !shape_valid(sh) || !shape_supported(sh, dtype)) return 0;
    return workspace_need(sh, dtype, want_grads != 0, from_boundary(*options),
                          options->head_evaluation == PCM_HEAD_COMPOSED);
}

namespace {

int run_actor_step(const void* hidden, const uint8_t* tokens, const float* logp_old, const float* adv,
                   const int32_t* kept_idx, const int32_t* n_kept, int max_kept_chunks, int T, int N, int A, int d, int ff,
                   int V, int dtype, const void* Wg, const void* Wu, const void* Wd, const void* Wo, const LossOptions& opt,
                   bool composed,
                   float* loss_out, float* logp_out, float* dWg, float* dWu, float* dWd, float* dWo, void* dX,
                   float* stats_out, int n_stats, void* workspace, size_t workspace_bytes, void* stream) {
    if (!hidden || !tokens || !logp_old || !adv || !kept_idx || !n_kept || !Wg || !Wu || !Wd || !Wo || !loss_out)
        return PCM_EINVAL;
    const int n_grad = (dWg != nullptr) + (dWu != nullptr) + (dWd != nullptr) + (dWo != nullptr);
    if (n_grad != 0 && n_grad != 4) return PCM_EINVAL;
    ActorShape sh{max_kept_chunks, T, N, A, d, ff, V};
    if (!shape_valid(sh) || T < 1 || N < 1 || (int64_t)T * N >= (int64_t)1 << 31) return PCM_EINVAL;
    if (!(opt.eps_low >= 0.f) || !(opt.eps_high >= 0.f) || opt.loss_scale != opt.loss_scale ||
        opt.entropy_coef != opt.entropy_coef || opt.panel_rows < 0)
        return PCM_EINVAL;
    if (dtype != PCM_F32 && dtype != PCM_BF16) return PCM_EINVAL;
    if (!shape_supported(sh, dtype)) return PCM_EUNSUPPORTED;
    const bool bwd = n_grad == 4 || dX != nullptr;
    if (opt.packed_weights != nullptr) {
        if (reinterpret_cast<uintptr_t>(opt.packed_weights) & 255u) return PCM_EINVAL;
        if (dtype != PCM_BF16 || composed) return PCM_EUNSUPPORTED;
    }
    if (opt.grad_sumsq_out != nullptr) {
        if (reinterpret_cast<uintptr_t>(opt.grad_sumsq_out) & 7u) return PCM_EINVAL;
        if (dtype != PCM_BF16 || composed || n_grad != 4) return PCM_EUNSUPPORTED;
    }
    // the split-precision forward pass of the per-chunk ratio exists for the evaluation as written only
    if (dtype == PCM_BF16 && opt.chunk_ratio && composed) return PCM_EUNSUPPORTED;
    const size_t need = workspace_need(sh, dtype, bwd, opt, composed);
    if (!workspace_ok(workspace, workspace_bytes, need)) return PCM_EWORKSPACE;

    ActorIO io{hidden, tokens, logp_old, adv, kept_idx, n_kept, Wg, Wu, Wd, Wo, opt,
               loss_out, logp_out, dWg, dWu, dWd, dWo, dX, stats_out, n_stats, composed};
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dtype == PCM_F32 ? actor_f32_run(sh, io, workspace, s) : actor_bf16_run(sh, io, workspace, s);
}

}  // namespace

extern "C" int grpo_masked_actor_step(const void* hidden, const uint8_t* tokens, const float* logp_old,
                                      const float* adv, const int32_t* kept_idx, const int32_t* n_kept,
                                      int max_kept_chunks, int T, int N, int A, int d, int ff, int V, int dtype,
                                      const void* Wg, const void* Wu, const void* Wd, const void* Wo,
                                      float eps_low, float eps_high, float loss_scale, float* loss_out,
                                      float* logp_out, float* dWg, float* dWu, float* dWd, float* dWo, void* dX,
                                      float* stats_out, void* workspace, size_t workspace_bytes, void* stream) {
    const LossOptions opt = plain_options(eps_low, eps_high, loss_scale);
    return run_actor_step(hidden, tokens, logp_old, adv, kept_idx, n_kept, max_kept_chunks, T, N, A, d, ff, V, dtype, Wg,
                          Wu, Wd, Wo, opt, false, loss_out, logp_out, dWg, dWu, dWd, dWo, dX, stats_out, 4, workspace,
                          workspace_bytes, stream);
}

extern "C" int grpo_masked_actor_step_ex(const void* hidden, const uint8_t* tokens, const float* logp_old,
                                         const float* adv, const int32_t* kept_idx, const int32_t* n_kept,
                                         int max_kept_chunks, int T, int N, int A, int d, int ff, int V, int dtype,
                                         const void* Wg, const void* Wu, const void* Wd, const void* Wo,
                                         const pcm_loss_options* options, float* loss_out, float* logp_out, float* dWg,
                                         float* dWu, float* dWd, float* dWo, void* dX, float* stats_out,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    if (!options) return PCM_EINVAL;
    if ((options->normalisation != PCM_NORM_SCALE && options->normalisation != PCM_NORM_TOKEN_MEAN) ||
        (options->ratio_level != PCM_RATIO_TOKEN && options->ratio_level != PCM_RATIO_CHUNK) ||
        (options->head_evaluation != PCM_HEAD_AS_WRITTEN && options->head_evaluation != PCM_HEAD_COMPOSED))
        return PCM_EINVAL;
    const LossOptions opt = from_boundary(*options);
    return run_actor_step(hidden, tokens, logp_old, adv, kept_idx, n_kept, max_kept_chunks, T, N, A, d, ff, V, dtype, Wg,
                          Wu, Wd, Wo, opt, options->head_evaluation == PCM_HEAD_COMPOSED, loss_out, logp_out, dWg, dWu,
                          dWd, dWo, dX, stats_out, 5, workspace, workspace_bytes, stream);
}

extern "C" size_t pcm_packed_head_bytes(int d, int ff, int V) {
    ActorShape sh{1, 1, 1, 1, d, ff, V};
    if (d < 1 || ff < 1 || V < 1 || !shape_supported(sh, PCM_BF16)) return 0;
    return packed_head_bytes(d, ff, V);
}

extern "C" int pcm_pack_head_weights(const void* Wg, const void* Wu, const void* Wd, const void* Wo, int d, int ff, int V,
                                     void* packed, void* stream) {
    if (!Wg || !Wu || !Wd || !Wo || !packed || d < 1 || ff < 1 || V < 1) return PCM_EINVAL;
    if (reinterpret_cast<uintptr_t>(packed) & 255u) return PCM_EINVAL;
    ActorShape sh{1, 1, 1, 1, d, ff, V};
    if (!shape_supported(sh, PCM_BF16)) return PCM_EUNSUPPORTED;
    return pack_head_weights(Wg, Wu, Wd, Wo, d, ff, V, packed, static_cast<hipStream_t>(stream));
}
