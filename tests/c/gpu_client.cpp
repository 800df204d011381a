// A client of the C boundary that uses nothing but the HIP runtime for memory: one training step of Algorithm 1
// (score, keep probabilities, sampling, masked actor step in bf16) on inputs made from a counter hash, results
// printed as one JSON line.  tests/test_gpu_c_client.py builds the same inputs in numpy, runs the same step through
// the Python binding and the CPU checker, and compares.  Built by paper_2605_16154_amd/build.py (hipcc, linked
// against libpcm.so); not part of the library.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pcm.h"

#define HIP_OK(x)                                                                         \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            std::fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define PCM_OK_OR_FAIL(x)                                                                 \
    do {                                                                                  \
        int r_ = (x);                                                                     \
        if (r_ != PCM_OK) {                                                               \
            std::fprintf(stderr, "%s at line %d\n", pcm_status_string(r_), __LINE__);     \
            return 3;                                                                     \
        }                                                                                 \
    } while (0)

// value in [-0.5, 0.5) from (stream, index): the top 24 bits of a multiplicative hash
static float unit(uint32_t stream, uint64_t i) {
    uint32_t x = (uint32_t)(i * 2654435761ull) ^ (stream * 0x9E3779B9u);
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return (float)(x >> 8) / 16777216.0f - 0.5f;
}
static uint16_t to_bf16(float f) {   // round to nearest even
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (uint16_t)u;
}

template <typename T>
static int upload(const std::vector<T>& h, T** d) {
    HIP_OK(hipMalloc(reinterpret_cast<void**>(d), h.size() * sizeof(T)));
    HIP_OK(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return 0;
}

int main() {
    const int n_groups = 2, G = 4, T = n_groups * G, N = 8, A = 56, K = 3, B = 4, d = 256, ff = 256, V = 256;
    const int max_kept = T * B;
    const int64_t rows_all = (int64_t)T * N * A;

    std::vector<float> actions((size_t)T * N * A);
    for (size_t i = 0; i < actions.size(); ++i) actions[i] = 2.0f * unit(1, i);
    std::vector<uint8_t> phase((size_t)T * N), reward(T), tokens((size_t)rows_all);
    for (int i = 0; i < T; ++i)
        for (int k = 0; k < N; ++k) phase[(size_t)i * N + k] = (uint8_t)(k * K / N);
    for (int i = 0; i < T; ++i) reward[i] = (uint8_t)((i % G) < 2 ? 1 : 0);        // two successes per group
    for (int i = 0; i < T; ++i)                                                      // successes act differently in phase 1
        if (reward[i])
            for (int k = 0; k < N; ++k)
                if (phase[(size_t)i * N + k] == 1)
                    for (int j = 0; j < A; ++j) actions[((size_t)i * N + k) * A + j] += 0.25f;
    for (size_t i = 0; i < tokens.size(); ++i) tokens[i] = (uint8_t)((unit(2, i) + 0.5f) * 256.0f);
    std::vector<uint16_t> hidden((size_t)rows_all * d), Wg((size_t)d * ff), Wu((size_t)d * ff), Wd((size_t)ff * d),
        Wo((size_t)d * V);
    for (size_t i = 0; i < hidden.size(); ++i) hidden[i] = to_bf16(2.0f * unit(3, i));
    for (size_t i = 0; i < Wg.size(); ++i) Wg[i] = to_bf16(0.15f * unit(4, i));
    for (size_t i = 0; i < Wu.size(); ++i) Wu[i] = to_bf16(0.15f * unit(5, i));
    for (size_t i = 0; i < Wd.size(); ++i) Wd[i] = to_bf16(0.15f * unit(6, i));
    for (size_t i = 0; i < Wo.size(); ++i) Wo[i] = to_bf16(0.15f * unit(7, i));
    std::vector<float> logp_old((size_t)rows_all);
    for (size_t i = 0; i < logp_old.size(); ++i) logp_old[i] = -5.545f + 0.6f * unit(8, i);   // around log(1 / 256)

    float *d_actions, *d_logp_old;
    uint8_t *d_phase, *d_reward, *d_tokens;
    uint16_t *d_hidden, *d_Wg, *d_Wu, *d_Wd, *d_Wo;
    if (upload(actions, &d_actions) || upload(logp_old, &d_logp_old) || upload(phase, &d_phase) || upload(reward, &d_reward) ||
        upload(tokens, &d_tokens) || upload(hidden, &d_hidden) || upload(Wg, &d_Wg) || upload(Wu, &d_Wu) || upload(Wd, &d_Wd) ||
        upload(Wo, &d_Wo))
        return 2;

    // outputs and scratch
    double *d_C, *d_p;
    uint8_t *d_valid, *d_active;
    float *d_adv, *d_loss, *d_logp, *d_dWg, *d_dWu, *d_dWd, *d_dWo, *d_stats;
    int32_t *d_kept, *d_off, *d_nk;
    void *d_state, *d_dX, *ws_score = nullptr, *ws_sample = nullptr, *ws_actor = nullptr;
    HIP_OK(hipMalloc((void**)&d_C, K * 8)); HIP_OK(hipMalloc((void**)&d_p, K * 8));
    HIP_OK(hipMalloc((void**)&d_valid, K)); HIP_OK(hipMalloc((void**)&d_active, T));
    HIP_OK(hipMalloc((void**)&d_adv, T * 4)); HIP_OK(hipMalloc((void**)&d_loss, 4));
    HIP_OK(hipMalloc((void**)&d_logp, (size_t)max_kept * A * 4)); HIP_OK(hipMalloc((void**)&d_stats, 4 * 4));
    HIP_OK(hipMalloc((void**)&d_dWg, (size_t)d * ff * 4)); HIP_OK(hipMalloc((void**)&d_dWu, (size_t)d * ff * 4));
    HIP_OK(hipMalloc((void**)&d_dWd, (size_t)ff * d * 4)); HIP_OK(hipMalloc((void**)&d_dWo, (size_t)d * V * 4));
    HIP_OK(hipMalloc((void**)&d_kept, max_kept * 4)); HIP_OK(hipMalloc((void**)&d_off, (T + 1) * 4));
    HIP_OK(hipMalloc((void**)&d_nk, 4)); HIP_OK(hipMalloc(&d_state, pcm_state_bytes(K)));
    HIP_OK(hipMalloc(&d_dX, (size_t)max_kept * A * d * 2));
    const size_t n_score = pcm_score_phases_workspace_bytes(n_groups, G, N, A, K);
    const size_t n_sample = pcm_sample_chunks_workspace_bytes(T, N, K, B);
    const size_t n_actor = grpo_masked_actor_step_workspace_bytes(max_kept, A, d, ff, V, PCM_BF16, 1);
    if (n_score == 0 || n_actor == 0) return 4;
    HIP_OK(hipMalloc(&ws_score, n_score));
    if (n_sample) HIP_OK(hipMalloc(&ws_sample, n_sample));
    HIP_OK(hipMalloc(&ws_actor, n_actor));

    hipStream_t s;
    HIP_OK(hipStreamCreate(&s));
    PCM_OK_OR_FAIL(pcm_state_init(d_state, K, s));
    PCM_OK_OR_FAIL(pcm_score_phases(d_actions, d_phase, d_reward, nullptr, n_groups, G, N, A, K, 1e-6, d_C, d_valid, d_adv,
                                    d_active, ws_score, n_score, s));
    PCM_OK_OR_FAIL(pcm_update_keep_probs(d_state, d_C, d_valid, K, 0.1, 5, d_p, s));
    PCM_OK_OR_FAIL(pcm_sample_chunks(d_p, d_phase, nullptr, d_active, T, N, K, B, 77, 0, d_kept, d_off, d_nk, ws_sample,
                                     n_sample, s));
    PCM_OK_OR_FAIL(grpo_masked_actor_step(d_hidden, d_tokens, d_logp_old, d_adv, d_kept, d_nk, max_kept, T, N, A, d, ff, V,
                                          PCM_BF16, d_Wg, d_Wu, d_Wd, d_Wo, 0.2f, 0.4f, 1.0f / T, d_loss, d_logp, d_dWg,
                                          d_dWu, d_dWd, d_dWo, d_dX, d_stats, ws_actor, n_actor, s));
    HIP_OK(hipStreamSynchronize(s));

    double C[K], p[K];
    float loss, stats[4];
    int32_t nk;
    std::vector<int32_t> kept(max_kept);
    std::vector<float> dWo((size_t)d * V), dWg((size_t)d * ff);
    HIP_OK(hipMemcpy(C, d_C, sizeof C, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(p, d_p, sizeof p, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&loss, d_loss, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(stats, d_stats, sizeof stats, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&nk, d_nk, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(kept.data(), d_kept, kept.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dWo.data(), d_dWo, dWo.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dWg.data(), d_dWg, dWg.size() * 4, hipMemcpyDeviceToHost));
    double sq_o = 0.0, sq_g = 0.0;
    for (float x : dWo) sq_o += (double)x * x;
    for (float x : dWg) sq_g += (double)x * x;

    std::printf("{\"C\": [");
    for (int c = 0; c < K; ++c) std::printf("%s%.17g", c ? ", " : "", C[c]);
    std::printf("], \"p\": [");
    for (int c = 0; c < K; ++c) std::printf("%s%.17g", c ? ", " : "", p[c]);
    std::printf("], \"n_kept\": %d, \"kept\": [", nk);
    for (int q = 0; q < nk; ++q) std::printf("%s%d", q ? ", " : "", kept[q]);
    std::printf("], \"loss\": %.9g, \"clip_fraction\": %.9g, \"rows\": %.9g, \"dWo_sumsq\": %.17g, \"dWg_sumsq\": %.17g}\n", loss,
                stats[0], stats[3], sq_o, sq_g);
    return 0;
}
