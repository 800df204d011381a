// pcm_label_phases: the deterministic gripper-based phase label of every chunk (App. D, phase
// allotment rules), the step that produces the `phase` input of the selection calls.
//
// One workgroup per trajectory.  Pass 1: the threads stride over the trajectory's timesteps (one
// strided load each, several in flight per thread), test the gripper value against the close
// threshold and add the hits to per-chunk counters in LDS.  Pass 2: every chunk looks at the
// counts of its three neighbours on either side and at the index of the trajectory's last
// sustained-close chunk (a workgroup maximum), and applies the rules in priority order.  All
// threshold tests are integer comparisons of the count against the chunk length (g_f >= 0.75 is
// 4 n >= 3 L, and so on).
#include "common.h"

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr int kBatch = 8;                               // timesteps a thread requests at a time

enum : uint8_t { kApproach = 0, kPreGrasp = 1, kActiveGrip = 2, kReleaseRamp = 3, kTail = 4 };

__global__ __launch_bounds__(kThreads) void label_phases(const float* __restrict__ actions,
                                                         const int32_t* __restrict__ n_chunks, int N, int L, int D,
                                                         int gripper_dim, float close_threshold,
                                                         uint8_t* __restrict__ phase) {
    extern __shared__ int lds_counts[];                 // [N] close timesteps per chunk, then the last grasp chunk
    int* count = lds_counts;
    int* last_grasp = lds_counts + N;
    const int i = blockIdx.x, tid = threadIdx.x;
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni < 0 ? 0 : (Ni > N ? N : Ni);
    for (int j = tid; j < N; j += kThreads) count[j] = 0;
    if (tid == 0) *last_grasp = -1;
    __syncthreads();

    const float* traj = actions + (size_t)i * N * L * D + gripper_dim;
    const int steps = Ni * L;                           // timestep e of the trajectory is row e of [N * L, D]
    for (int e0 = tid; e0 < steps; e0 += kBatch * kThreads) {
        float g[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int e = e0 + u * kThreads;
            g[u] = e < steps ? traj[(size_t)e * D] : close_threshold;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int e = e0 + u * kThreads;
            if (e < steps && g[u] > close_threshold) atomicAdd(&count[e / L], 1);
        }
    }
    __syncthreads();
    for (int j = tid; j < Ni; j += kThreads)
        if (4 * count[j] >= 3 * L) atomicMax(last_grasp, j);
    __syncthreads();
    const int last = *last_grasp;

    uint8_t* out = phase + (size_t)i * N;
    for (int j = tid; j < N; j += kThreads) {
        uint8_t label = kApproach;
        if (j < Ni) {
            const int n = count[j];
            bool before_grasp = false, after_grasp = false;
#pragma unroll
            for (int d = 1; d <= 3; ++d) {
                if (j + d < Ni) before_grasp |= 4 * count[j + d] >= 3 * L;
                if (j - d >= 0) after_grasp |= 4 * count[j - d] >= 3 * L;
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
    label_phases<<<(unsigned)T, kThreads, ((size_t)N + 1) * sizeof(int), s>>>(actions, n_chunks, N, L, D, gripper_dim,
                                                                            close_threshold, phase);
    return launch_status();
}
