// pcm_score_phases: group-relative advantages (Eq. 1) and the batch phase score C_c (Eq. 5).
//
// Four launches on the caller's stream:
//   prepare     zero the integer accumulators; one thread per trajectory writes advantage/active
//   accumulate  streaming pass over the action tensor: every workgroup owns a slice of one
//               trajectory's chunks, keeps per-phase 64-bit integer sums in LDS and adds the
//               phases it met to the group's accumulators with 64-bit global atomics
//   pairs       one wavefront per (group, phase): difference of pooled means, squared terms in
//               parallel, added in index order by one lane, square root
//   mean        one lane per phase: mean of the pair scores over contributing groups
//
// The action pass is bandwidth-bound (224 B per chunk plus one phase byte); everything after it
// touches a few KB.  Integer accumulation makes the sums independent of slice and arrival order,
// which is what lets the sampler downstream be reproduced bit for bit.
//
// This file must be compiled without floating-point contraction: the fp64 tail is specified as
// separate multiplies and adds.
#include <mutex>

#include "common.h"

#pragma clang fp contract(off)

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr float kActionScale = 16777216.0f;                 // 2^24
constexpr double kActionUnscale = 1.0 / 16777216.0;         // 2^-24

using ull = unsigned long long;

struct ScoreWorkspace {
    ull* sums;            // [n_groups][2][K][A] integer sums of rint(a * 2^24); outcome 1 = success
    int* counts;          // [n_groups][2][K] chunks pooled
    double* pair;         // [n_groups][K] per-(group, phase) score
    uint8_t* pair_valid;  // [n_groups][K]
    size_t zero_words;    // 32-bit words to clear at the start (sums + counts are contiguous)
    size_t bytes;
};

ScoreWorkspace carve(void* ws, int n_groups, int A, int K) {
    Carver c(ws);
    ScoreWorkspace w;
    const size_t n_sum = (size_t)n_groups * 2 * K * A;
    const size_t n_cnt = (size_t)n_groups * 2 * K;
    w.sums = c.take<ull>(n_sum);
    const size_t after_sums = c.used();
    w.counts = c.take<int>(n_cnt);
    w.zero_words = (after_sums + n_cnt * sizeof(int) + 3) / 4;
    w.pair = c.take<double>((size_t)n_groups * K);
    w.pair_valid = c.take<uint8_t>((size_t)n_groups * K);
    w.bytes = c.used();
    return w;
}

__global__ __launch_bounds__(kThreads) void score_prepare(uint32_t* zero, size_t zero_words,
                                                          const uint8_t* __restrict__ reward, int T,
                                                          int G, double adv_eps, float* adv_out,
                                                          uint8_t* active_out) {
    const size_t gid = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t w = gid; w < zero_words; w += stride) zero[w] = 0u;
    for (size_t i = gid; i < (size_t)T; i += stride) {
        const int g = (int)(i / G);
        int s = 0;
        for (int r = 0; r < G; ++r) s += reward[(size_t)g * G + r] != 0;
        float a = 0.f;
        uint8_t act = 0;
        if (s != 0 && s != G) {
            const double mu = (double)s / (double)G;
            const double sigma = sqrt(mu * (1.0 - mu));
            const double r = reward[i] != 0 ? 1.0 : 0.0;
            a = (float)((r - mu) / (sigma + adv_eps));
            act = 1;
        }
        if (adv_out) adv_out[i] = a;
        if (active_out) active_out[i] = act;
    }
}

template <int VEC>
struct ActionVec;
template <>
struct ActionVec<4> {
    float v[4];
    __device__ void load(const float* p) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
};
template <>
struct ActionVec<1> {
    float v[1];
    __device__ void load(const float* p) { v[0] = *p; }
};

// grid = T * slices * phase_blocks workgroups; a workgroup pools the phases [c0, c0 + Kb) of its
// chunks (phase_blocks is 1 unless K*A sums do not fit in LDS; then the chunks are read once per
// block of phases).  LDS: Kb*A 64-bit sums followed by Kb chunk counts, indexed by phase - c0.
template <int VEC>
__global__ __launch_bounds__(kThreads) void score_accumulate(
    const float* __restrict__ actions, const uint8_t* __restrict__ phase,
    const uint8_t* __restrict__ reward, const int32_t* __restrict__ n_chunks, int G, int N, int A,
    int K, int Kb, int slices, ull* sums, int* counts) {
    extern __shared__ ull lds_sum[];
    int* lds_cnt = reinterpret_cast<int*>(lds_sum + (size_t)Kb * A);

    const int phase_blocks = (K + Kb - 1) / Kb;
    const int c0 = (blockIdx.x % phase_blocks) * Kb;
    const int kb = min(Kb, K - c0);                     // phases of this workgroup
    const int slice = (blockIdx.x / phase_blocks) % slices;
    const int i = blockIdx.x / phase_blocks / slices;
    const int g = i / G;
    int s = 0;
    for (int r = 0; r < G; ++r) s += reward[(size_t)g * G + r] != 0;
    if (s == 0 || s == G) return;  // uniform rewards: the group has no score (whole workgroup exits)
    const int outcome = reward[i] != 0;
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni < 0 ? 0 : (Ni > N ? N : Ni);
    const int per = (N + slices - 1) / slices;
    const int k0 = slice * per;
    const int k1 = min(Ni, k0 + per);
    if (k0 >= k1) return;

    const int tid = threadIdx.x;
    for (int e = tid; e < kb * A; e += kThreads) lds_sum[e] = 0;
    for (int c = tid; c < kb; c += kThreads) lds_cnt[c] = 0;
    __syncthreads();

    const int AV = A / VEC;            // vectors per chunk
    const int CPI = kThreads / AV;     // chunks per pass of the workgroup
    const int jv = tid % AV, cs = tid / AV;
    if (cs < CPI) {
        long long acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0;
        int cur = -1, run = 0;
        auto flush = [&]() {
            if (cur >= 0 && cur < kb && run > 0) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    atomicAdd(&lds_sum[(size_t)cur * A + jv * VEC + v], (ull)acc[v]);
                if (jv == 0) atomicAdd(&lds_cnt[cur], run);
            }
        };
        const float* row = actions + (size_t)i * N * A + (size_t)jv * VEC;
        const uint8_t* ph = phase + (size_t)i * N;
        for (int k = k0 + cs; k < k1; k += CPI) {
            const int c = min((int)ph[k], K - 1) - c0;  // ids beyond the last phase count as the last; outside [0, kb): another block's
            ActionVec<VEC> x;
            x.load(row + (size_t)k * A);
            if (c != cur) {
                flush();
                cur = c;
                run = 0;
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = 0;
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += __float2ll_rn(x.v[v] * kActionScale);
            ++run;
        }
        flush();
    }
    __syncthreads();

    const size_t base = ((size_t)g * 2 + outcome) * K + c0;
    for (int e = tid; e < kb * A; e += kThreads) {
        const int c = e / A;
        if (lds_cnt[c] > 0) atomicAdd(&sums[base * A + e], lds_sum[e]);
    }
    for (int c = tid; c < kb; c += kThreads)
        if (lds_cnt[c] > 0) atomicAdd(&counts[base + c], lds_cnt[c]);
}

// One wavefront per (group, phase).  All threads reach both barriers.
__global__ __launch_bounds__(kThreads) void score_pairs(const ull* __restrict__ sums,
                                                        const int* __restrict__ counts, int n_groups,
                                                        int A, int K, double* pair,
                                                        uint8_t* pair_valid) {
    __shared__ double sq[kThreads / kWave][256];
    const int wv = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int w = blockIdx.x * (kThreads / kWave) + wv;
    const bool in_range = w < n_groups * K;
    int n_pos = 0, n_neg = 0;
    size_t pos_base = 0, neg_base = 0;
    if (in_range) {
        const int g = w / K, c = w % K;
        pos_base = ((size_t)g * 2 + 1) * K + c;
        neg_base = ((size_t)g * 2 + 0) * K + c;
        n_pos = counts[pos_base];
        n_neg = counts[neg_base];
    }
    const bool ok = in_range && n_pos > 0 && n_neg > 0;
    if (ok) {
        const double dp = (double)n_pos, dn = (double)n_neg;
        for (int j = lane; j < A; j += kWave) {
            const double mp = (double)(long long)sums[pos_base * A + j] / dp;
            const double mn = (double)(long long)sums[neg_base * A + j] / dn;
            const double diff = mp - mn;
            sq[wv][j] = diff * diff;
        }
    }
    __syncthreads();
    if (in_range && lane == 0) {
        if (ok) {
            double acc = 0.0;
            for (int j = 0; j < A; ++j) acc = acc + sq[wv][j];
            pair[w] = sqrt(acc) * kActionUnscale;
            pair_valid[w] = 1;
        } else {
            pair[w] = 0.0;
            pair_valid[w] = 0;
        }
    }
}

// Batch score of phase c = mean over the groups that contributed, added for g ascending (the order is
// part of the definition: the result must not depend on the launch).  One workgroup: the per-group values
// are brought into LDS a block of groups at a time (kMeanEntries values, so 4096 / K groups) with coalesced
// loads, then lane c adds its column in order.
constexpr int kMeanEntries = 4096;
__global__ __launch_bounds__(256) void score_mean(const double* __restrict__ pair, const uint8_t* __restrict__ pair_valid,
                                                  int n_groups, int K, double* C_out, uint8_t* valid_out) {
    __shared__ double val[kMeanEntries];
    __shared__ uint8_t ok[kMeanEntries];
    const int c = threadIdx.x;
    const int block_groups = kMeanEntries / K;          // K <= 64: at least 64 groups
    double tot = 0.0;
    int n = 0;
    for (int g0 = 0; g0 < n_groups; g0 += block_groups) {
        const int groups = min(block_groups, n_groups - g0);
        // eight loads per thread in flight before the first is stored (a thread has at most 16 entries per block)
        for (int i0 = threadIdx.x; i0 < groups * K; i0 += 8 * 256) {
            double v[8];
            uint8_t o[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * 256;
                v[u] = i < groups * K ? pair[(size_t)g0 * K + i] : 0.0;
                o[u] = i < groups * K ? pair_valid[(size_t)g0 * K + i] : 0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * 256;
                if (i < groups * K) {
                    val[i] = o[u] ? v[u] : 0.0;   // a skipped pair adds +0.0, which leaves the non-negative sum as it is
                    ok[i] = o[u];
                }
            }
        }
        __syncthreads();
        if (c < K) {
            // branch-free, so that the LDS reads run ahead of the additions, which stay in group order
#pragma unroll 8
            for (int g = 0; g < groups; ++g) {
                tot = tot + val[g * K + c];
                n += ok[g * K + c];
            }
        }
        __syncthreads();
    }
    if (c < K) {
        C_out[c] = n > 0 ? tot / (double)n : 0.0;
        valid_out[c] = n > 0 ? 1 : 0;
    }
}

bool shape_ok(int n_groups, int G, int N, int A, int K) {
    return n_groups >= 1 && G >= 1 && N >= 1 && A >= 1 && A <= 256 && K >= 1 && K <= PCM_MAX_PHASES &&
           (int64_t)n_groups * G * N < (int64_t)1 << 31;
}

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" size_t pcm_score_phases_workspace_bytes(int n_groups, int G, int N, int A, int K) {
    if (!shape_ok(n_groups, G, N, A, K)) return 0;
    return carve(nullptr, n_groups, A, K).bytes;
}

// ---- scratch memory owned by the library, for the entry point that takes no workspace -------------
// Every GPU holds its own copy of this array at its own address.  In host code the array's name is
// only a handle for hipGetSymbolAddress: the address that kernels and fills receive is the one that
// call returns on the device that is current, looked up once per device and kept.
constexpr size_t kStaticScratchBytes = PCM_SCORE_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Argument checks and the four launches shared by both entry points; `workspace` has been checked
// to hold carve(...).bytes.
int run_score(const float* actions, const uint8_t* phase, const uint8_t* reward, const int32_t* n_chunks,
              int n_groups, int G, int N, int A, int K, double adv_eps, double* C_out, uint8_t* valid_out,
              float* adv_out, uint8_t* active_out, const ScoreWorkspace& w, hipStream_t s) {
    // phases per workgroup: all K if their sums fit in 64 KB of LDS (A <= 256: at least 31 do)
    int Kb = (int)((size_t)64 * 1024 / ((size_t)A * sizeof(ull) + sizeof(int)));
    if (Kb > K) Kb = K;
    const int phase_blocks = ceil_div(K, Kb);
    const size_t lds_bytes = (size_t)Kb * A * sizeof(ull) + (size_t)Kb * sizeof(int);
    const int T = n_groups * G;
    {
        StageTimer t(ST_SCORE_PREPARE, s);
        const size_t work = w.zero_words > (size_t)T ? w.zero_words : (size_t)T;
        const int blocks = (int)((work + kThreads - 1) / kThreads);
        score_prepare<<<blocks < 1024 ? blocks : 1024, kThreads, 0, s>>>(
            reinterpret_cast<uint32_t*>(w.sums), w.zero_words, reward, T, G, adv_eps, adv_out,
            active_out);
    }
    {
        StageTimer t(ST_SCORE_ACCUMULATE, s);
        const bool vec4 = (A % 4 == 0) && ((reinterpret_cast<uintptr_t>(actions) & 15u) == 0);
        const int chunks_per_pass = kThreads / (vec4 ? A / 4 : A);
        // enough workgroups to cover the chip several times over, but at least two passes each
        int slices = ceil_div(2048, T);
        const int max_slices = ceil_div(N, 2 * chunks_per_pass);
        if (slices > max_slices) slices = max_slices;
        if (slices < 1) slices = 1;
        const unsigned grid = (unsigned)T * (unsigned)slices * (unsigned)phase_blocks;
        if (vec4)
            score_accumulate<4><<<grid, kThreads, lds_bytes, s>>>(actions, phase, reward, n_chunks, G,
                                                                N, A, K, Kb, slices, w.sums, w.counts);
        else
            score_accumulate<1><<<grid, kThreads, lds_bytes, s>>>(actions, phase, reward, n_chunks, G,
                                                                N, A, K, Kb, slices, w.sums, w.counts);
    }
    {
        StageTimer t(ST_SCORE_FINALISE, s);
        const int waves = n_groups * K;
        score_pairs<<<ceil_div(waves, kThreads / kWave), kThreads, 0, s>>>(w.sums, w.counts, n_groups, A,
                                                                         K, w.pair, w.pair_valid);
        score_mean<<<1, 256, 0, s>>>(w.pair, w.pair_valid, n_groups, K, C_out, valid_out);
    }
    return launch_status();
}

bool args_ok(const float* actions, const uint8_t* phase, const uint8_t* reward, int n_groups, int G, int N, int A,
             int K, double adv_eps, const double* C_out, const uint8_t* valid_out) {
    return actions && phase && reward && C_out && valid_out && shape_ok(n_groups, G, N, A, K) && adv_eps >= 0.0;
}

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void* scratch_of_device[kMaxDevices] = {};

int static_scratch(void** out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return PCM_EHIP;
    if (device < 0 || device >= kMaxDevices) return PCM_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (scratch_of_device[device] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return PCM_EHIP;
        }
        scratch_of_device[device] = p;
    }
    *out = scratch_of_device[device];
    return PCM_OK;
}

}  // namespace

extern "C" int pcm_score_phases(const float* actions, const uint8_t* phase, const uint8_t* reward,
                                const int32_t* n_chunks, int n_groups, int G, int N, int A, int K,
                                double adv_eps, double* C_out, uint8_t* valid_out, float* adv_out,
                                uint8_t* active_out, void* workspace, size_t workspace_bytes,
                                void* stream) {
    if (!args_ok(actions, phase, reward, n_groups, G, N, A, K, adv_eps, C_out, valid_out)) return PCM_EINVAL;
    ScoreWorkspace w = carve(workspace, n_groups, A, K);
    if (!workspace_ok(workspace, workspace_bytes, w.bytes)) return PCM_EWORKSPACE;
    return run_score(actions, phase, reward, n_chunks, n_groups, G, N, A, K, adv_eps, C_out, valid_out, adv_out,
                     active_out, w, static_cast<hipStream_t>(stream));
}

extern "C" int pcm_score_phases_static(const float* actions, const uint8_t* phase, const uint8_t* reward,
                                       const int32_t* n_chunks, int n_groups, int G, int N, int A, int K,
                                       double adv_eps, double* C_out, uint8_t* valid_out, float* adv_out,
                                       uint8_t* active_out, void* stream) {
    if (!args_ok(actions, phase, reward, n_groups, G, N, A, K, adv_eps, C_out, valid_out)) return PCM_EINVAL;
    if (carve(nullptr, n_groups, A, K).bytes > kStaticScratchBytes) return PCM_EWORKSPACE;
    void* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != PCM_OK) return rc;
    const ScoreWorkspace w = carve(base, n_groups, A, K);
    return run_score(actions, phase, reward, n_chunks, n_groups, G, N, A, K, adv_eps, C_out, valid_out, adv_out,
                     active_out, w, static_cast<hipStream_t>(stream));
}
