// pcm_state_init / pcm_update_keep_probs: score buffers and keep probabilities (Eq. 7-9).
//
// The state is K <= 64 numbers; one lane walks it in index order so the arithmetic has a single,
// written-down order.  The buffers of Eq. 7 are held as running sums S_c (Eq. 8 only sums them).
// The refresh trigger counts appended steps (Sec. 4.3: first batch, then every T_rc steps).
#include "common.h"

#pragma clang fp contract(off)

namespace pcm {
namespace {

// Device view of the state block: int64 step; int64 since; double S[K]; int64 count[K]; double p[K].
struct StateView {
    long long* step;
    long long* since;
    double* S;
    long long* count;
    double* p;
    __host__ __device__ StateView(void* base, int K) {
        char* b = static_cast<char*>(base);
        step = reinterpret_cast<long long*>(b);
        since = reinterpret_cast<long long*>(b + 8);
        S = reinterpret_cast<double*>(b + 16);
        count = reinterpret_cast<long long*>(b + 16 + 8 * (size_t)K);
        p = reinterpret_cast<double*>(b + 16 + 16 * (size_t)K);
    }
};

__global__ void state_init(void* state, int K) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    StateView v(state, K);
    *v.step = 0;
    *v.since = 0;
    for (int c = 0; c < K; ++c) {
        v.S[c] = 0.0;
        v.count[c] = 0;
        v.p[c] = 1.0;
    }
}

// One wavefront, lane c owns phase c (K <= 64).  Everything is per phase except the maximum of the
// sums, and a maximum does not depend on the order it is taken in, so the results are those of the
// one-lane walk in index order.
__global__ __launch_bounds__(kWave) void update_keep_probs(void* state, const double* __restrict__ C,
                                                            const uint8_t* __restrict__ valid, int K, double p_min,
                                                            int T_rc, double* keep_probs_out) {
    if (blockIdx.x != 0) return;
    StateView v(state, K);
    const int c = threadIdx.x;
    const bool mine = c < K;
    double S = 0.0, p = 0.0;
    long long count = 0;
    if (mine) {
        S = v.S[c];
        count = v.count[c];
        p = v.p[c];
        if (valid[c]) {
            S = S + C[c];                      // Eq. 7: append (as a running sum)
            count += 1;
        }
    }
    long long since = *v.since + 1;
    const long long step = *v.step;
    if (step == 0 || since == (long long)T_rc) {
        double s_max = (mine && S > 0.0) ? S : 0.0;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const double other = __shfl_xor(s_max, off, kWave);
            s_max = other > s_max ? other : s_max;
        }
        // Eq. 8: rho_c / max rho = S_c / max S (the share denominator cancels)
        const double rho_tilde = s_max > 0.0 ? S / s_max : 0.0;
        p = rho_tilde > p_min ? rho_tilde : p_min;   // Eq. 9
        S = 0.0;
        count = 0;
        since = 0;
    }
    __builtin_amdgcn_wave_barrier();           // every lane has read step and since before lane 0 rewrites them
    if (mine) {
        v.S[c] = S;
        v.count[c] = count;
        v.p[c] = p;
        if (keep_probs_out) keep_probs_out[c] = p;
    }
    if (c == 0) {
        *v.since = since;
        *v.step = step + 1;
    }
}

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" size_t pcm_state_bytes(int K) {
    if (K < 1 || K > PCM_MAX_PHASES) return 0;
    return 16 + 24 * (size_t)K;
}

extern "C" int pcm_state_init(void* state, int K, void* stream) {
    if (!state || K < 1 || K > PCM_MAX_PHASES) return PCM_EINVAL;
    if (reinterpret_cast<uintptr_t>(state) & 7u) return PCM_EINVAL;
    state_init<<<1, kWave, 0, static_cast<hipStream_t>(stream)>>>(state, K);
    return launch_status();
}

extern "C" int pcm_update_keep_probs(void* state, const double* C, const uint8_t* valid, int K,
                                     double p_min, int T_rc, double* keep_probs_out, void* stream) {
    if (!state || !C || !valid || K < 1 || K > PCM_MAX_PHASES) return PCM_EINVAL;
    if (reinterpret_cast<uintptr_t>(state) & 7u) return PCM_EINVAL;
    if (!(p_min > 0.0 && p_min <= 1.0) || T_rc < 1) return PCM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StageTimer t(ST_KEEP_PROBS, s);
    update_keep_probs<<<1, kWave, 0, s>>>(state, C, valid, K, p_min, T_rc, keep_probs_out);
    return launch_status();
}
