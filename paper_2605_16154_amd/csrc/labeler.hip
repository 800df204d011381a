// pcm_label_phases: the deterministic gripper-based phase label of every chunk (App. D, phase
// allotment rules), the step that produces the `phase` input of the selection calls.
//
// One wavefront per trajectory.  Pass 1: lanes stride over the chunks, count the timesteps whose
// gripper value exceeds the close threshold (L strided loads per chunk out of the chunk's L*D
// contiguous floats) and keep the counts in LDS.  Pass 2: every chunk looks at the counts of its
// three neighbours on either side and at the index of the trajectory's last sustained-close chunk
// (a wave maximum), and applies the rules in priority order.  All threshold tests are integer
// comparisons of the count against the chunk length (g_f >= 0.75 is 4 n >= 3 L, and so on).
#include "common.h"

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;

enum : uint8_t { kApproach = 0, kPreGrasp = 1, kActiveGrip = 2, kReleaseRamp = 3, kTail = 4 };

__global__ __launch_bounds__(kThreads) void label_phases(const float* __restrict__ actions,
                                                         const int32_t* __restrict__ n_chunks, int T, int N, int L,
                                                         int D, int gripper_dim, float close_threshold,
                                                         uint8_t* __restrict__ phase) {
    extern __shared__ uint16_t lds_counts[];            // [waves][N]
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int waves = blockDim.x / kWave;
    const int i = blockIdx.x * waves + wv;
    if (i >= T) return;                                 // no workgroup barrier below
    uint16_t* count = lds_counts + (size_t)wv * N;
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni < 0 ? 0 : (Ni > N ? N : Ni);
    const int A = L * D;
    const float* traj = actions + (size_t)i * N * A;
    int last = -1;                                      // last sustained-close chunk seen by this lane
    for (int j = lane; j < Ni; j += kWave) {
        const float* chunk = traj + (size_t)j * A + gripper_dim;
        int n = 0;
        for (int t = 0; t < L; ++t) n += chunk[t * D] > close_threshold ? 1 : 0;
        count[j] = (uint16_t)n;
        if (4 * n >= 3 * L) last = j;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off, kWave));
    __builtin_amdgcn_wave_barrier();
    uint8_t* out = phase + (size_t)i * N;
    for (int j = lane; j < N; j += kWave) {
        uint8_t label = kApproach;
        if (j < Ni) {
            const int n = count[j];
            bool before_grasp = false, after_grasp = false;
#pragma unroll
            for (int d = 1; d <= 3; ++d) {
                if (j + d < Ni) before_grasp |= 4 * (int)count[j + d] >= 3 * L;
                if (j - d >= 0) after_grasp |= 4 * (int)count[j - d] >= 3 * L;
            }
            if (2 * n >= L) label = kActiveGrip;
            else if (before_grasp && 10 * n >= L) label = kPreGrasp;
            else if (after_grasp) label = kReleaseRamp;
            else if (last < 0 || j < last) label = kApproach;
            else label = kTail;
        }
        out[j] = label;
    }
}

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" int pcm_label_phases(const float* actions, const int32_t* n_chunks, int T, int N, int L, int D,
                                int gripper_dim, float close_threshold, uint8_t* phase, void* stream) {
    if (!actions || !phase) return PCM_EINVAL;
    if (T < 1 || N < 1 || N > PCM_MAX_CHUNK_SLOTS || L < 1 || L > 4096 || D < 1 || gripper_dim < 0 || gripper_dim >= D ||
        close_threshold != close_threshold || (int64_t)T * N >= (int64_t)1 << 31)
        return PCM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StageTimer t(ST_LABEL_PHASES, s);
    const int waves = kWavesPerBlock;                   // N <= 4096: four count arrays of 2 N bytes are 32 KB at most
    label_phases<<<ceil_div(T, waves), waves * kWave, (size_t)waves * N * sizeof(uint16_t), s>>>(
        actions, n_chunks, T, N, L, D, gripper_dim, close_threshold, phase);
    return launch_status();
}
