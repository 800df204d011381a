// pcm_sample_chunks: fixed-budget weighted sampling without replacement (Eq. 10) and the
// compaction that expresses physical shrinking (Sec. 4.5; Algorithm 1, inner loop).
//
// One launch (two for very many trajectories and for the top-phase selector):
//   compact  one wavefront per trajectory.  The per-trajectory kept counts min(B, N_i) (0 if inactive)
//            are known before any draw, so every workgroup adds up the counts of the trajectories
//            before its own to find where its output starts (a few KB of reads; for more than
//            kFusedScanMax trajectories, and for the top-phase selector whose counts need a pass over
//            the phases, a separate one-workgroup scan kernel writes the offsets first).  Lanes own
//            contiguous runs of chunk slots with their integer weights in registers (in LDS when a
//            lane owns more than eight), an inclusive wave scan of lane sums is kept up to date
//            across the min(B, N_i) successive draws, then kept slots are written in ascending order
//            at the trajectory's offset (wave prefix of per-lane popcounts)
//
// All arithmetic after the weight quantisation is integer, and the random bits depend only on
// (seed, step, trajectory, round), so the kept set is a pure function of the inputs.
#include "common.h"

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kFusedScanMax = 4096;   // trajectories up to which every workgroup sums the earlier counts itself

// Philox-4x32, 10 rounds (Salmon et al., SC'11): multipliers and Weyl key increments as published.
constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

__device__ inline uint64_t philox_bits(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                       uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(kPhiloxM0, c0), lo0 = kPhiloxM0 * c0;
        const uint32_t hi1 = __umulhi(kPhiloxM1, c2), lo1 = kPhiloxM1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += kPhiloxW0; k1 += kPhiloxW1;
    }
    return (uint64_t)c0 | ((uint64_t)c1 << 32);
}

// Index of the largest keep probability, lowest index on ties (the one phase the "top phase"
// selector draws from).
__device__ inline int top_phase(const double* keep_probs, int K) {
    int best = 0;
    for (int c = 1; c < K; ++c)
        if (keep_probs[c] > keep_probs[best]) best = c;
    return best;
}

// Chunks a trajectory keeps: min(B, eligible chunks), 0 if inactive.  Every valid chunk is eligible
// except under the top-phase selector, where only chunks of phase `only` (>= 0) are.
__device__ inline int kept_count(const int32_t* n_chunks, const uint8_t* active, const uint8_t* phase, int i, int N,
                                 int K, int B, int only) {
    if (active && !active[i]) return 0;
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni < 0 ? 0 : (Ni > N ? N : Ni);
    if (only >= 0) {
        const uint8_t* ph = phase + (size_t)i * N;
        int n = 0;
        for (int k = 0; k < Ni; ++k) {
            int c = ph[k];
            c = c < K ? c : K - 1;
            n += c == only;
        }
        Ni = n;
    }
    return Ni < B ? Ni : B;
}

__device__ inline int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(v, d, kWave);
        if (lane >= d) v += up;
    }
    return v;
}

__global__ __launch_bounds__(kThreads) void sample_scan(const double* __restrict__ keep_probs,
                                                        const uint8_t* __restrict__ phase,
                                                        const int32_t* __restrict__ n_chunks,
                                                        const uint8_t* __restrict__ active, int T, int N, int K,
                                                        int B, int selector, int32_t* kept_offsets, int32_t* n_kept) {
    __shared__ int wave_total[kWavesPerBlock];
    const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
    const int only = selector == PCM_SELECT_TOP_PHASE ? top_phase(keep_probs, K) : -1;
    int carry = 0;
    for (int base = 0; base < T; base += kThreads) {
        const int i = base + tid;
        const int cnt = i < T ? kept_count(n_chunks, active, phase, i, N, K, B, only) : 0;
        const int incl = wave_inclusive_scan(cnt, lane);
        if (lane == kWave - 1) wave_total[wv] = incl;
        __syncthreads();
        int before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            if (w < wv) before += wave_total[w];
            all += wave_total[w];
        }
        if (i < T) kept_offsets[i] = carry + before + incl - cnt;
        carry += all;
        __syncthreads();
    }
    if (tid == 0) {
        kept_offsets[T] = carry;
        *n_kept = carry;
    }
}

// LDS: K quantised phase weights, then one N-entry weight array per wavefront.
// kRegs > 0: a lane owns at most kRegs chunk slots and keeps their weights in registers; kRegs == 0: any
// N, weights in LDS.  kFusedScan: the workgroup computes its own output offset (and writes kept_offsets,
// n_kept) instead of reading offsets written by sample_scan.
template <int kRegs, bool kFusedScan>
__global__ __launch_bounds__(kThreads) void sample_compact(
    const double* __restrict__ keep_probs, const uint8_t* __restrict__ phase,
    const int32_t* __restrict__ n_chunks, const uint8_t* __restrict__ active, int T, int N, int K, int B,
    int selector, uint64_t seed, uint64_t step, int32_t* kept_offsets, int32_t* n_kept, int32_t* kept_idx) {
    extern __shared__ uint32_t lds[];
    uint32_t* qtab = lds;
    const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
    // This lane's phase bytes are requested first (their address depends on the launch geometry only), so that they
    // travel while the weights table and the output offset are worked out.
    uint8_t my_phase[kRegs > 0 ? kRegs : 1];
    if (kRegs > 0) {
        const int i_early = blockIdx.x * (blockDim.x / kWave) + wv;
        const int per_lane_early = (N + kWave - 1) / kWave;
#pragma unroll
        for (int j = 0; j < kRegs; ++j) {
            const int k = lane * per_lane_early + j;
            my_phase[j] = (i_early < T && j < per_lane_early && k < N) ? phase[(size_t)i_early * N + k] : 0;
        }
    }
    uint32_t* w = lds + PCM_MAX_PHASES + (size_t)wv * (N + 2 * PCM_MAX_PHASES);
    int* n_in_phase = reinterpret_cast<int*>(w + N);      // stratified selector: chunks per phase, then budgets
    int* budget = n_in_phase + PCM_MAX_PHASES;

    const int waves_per_block = blockDim.x / kWave;
    const int only = selector == PCM_SELECT_TOP_PHASE ? top_phase(keep_probs, K) : -1;
    for (int c = tid; c < K; c += blockDim.x) {
        uint32_t q = 1u;                      // uniform selector: equal weights
        if (selector == PCM_SELECT_PCM || selector == PCM_SELECT_STRATIFIED) {
            const double x = keep_probs[c] * 65536.0 + 0.5;
            if (x >= 65536.0) q = 65536u;
            else if (x >= 1.0) q = (uint32_t)x;   // truncation = floor for positive x
        } else if (selector == PCM_SELECT_TOP_PHASE) {
            q = c == only ? 1u : 0u;
        }
        qtab[c] = q;
    }
    __syncthreads();

    const int i = blockIdx.x * waves_per_block + wv;
    const int m = i < T ? kept_count(n_chunks, active, phase, i, N, K, B, only) : 0;
    int offset = 0;
    if (kFusedScan) {
        // kept chunks of all trajectories before this workgroup's first, then of the earlier wavefronts
        __shared__ int part[kWavesPerBlock + 1][kWavesPerBlock];
        const int i0 = blockIdx.x * waves_per_block;
        int before = 0;
        if (n_chunks == nullptr && active == nullptr) {
            before = i0 * (N < B ? N : B);                                   // every trajectory keeps min(B, N)
        } else {
            int mine = 0;
            for (int j = tid; j < i0; j += blockDim.x) mine += kept_count(n_chunks, active, phase, j, N, K, B, -1);
#pragma unroll
            for (int off = kWave / 2; off > 0; off >>= 1) mine += __shfl_xor(mine, off, kWave);
            if (lane == 0) part[0][wv] = mine;
        }
        if (lane == 0) part[1][wv] = m;
        __syncthreads();
        if (!(n_chunks == nullptr && active == nullptr))
            for (int q = 0; q < waves_per_block; ++q) before += part[0][q];
        for (int q = 0; q < wv; ++q) before += part[1][q];
        offset = before;
        if (i < T && lane == 0) {
            kept_offsets[i] = offset;
            if (i == T - 1) {
                kept_offsets[T] = offset + m;
                *n_kept = offset + m;
            }
        }
    } else if (i < T) {
        offset = kept_offsets[i];
    }
    if (i >= T || m == 0) return;             // no workgroup barrier below this point
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni > N ? N : Ni;

    const int per_lane = (N + kWave - 1) / kWave;   // <= 64 because N <= 4096
    const int k_lo = lane * per_lane;
    const uint8_t* ph = phase + (size_t)i * N;
    auto phase_of = [&](int k) {
        const int c = ph[k];
        return c < K ? c : K - 1;
    };

    // Stratified selector: a fixed budget per phase, m shared out in proportion to N_c q_c by the largest-
    // remainder rule with caps N_c (lane c owns phase c), then uniform draws inside each phase.
    int passes = 1;
    if (selector == PCM_SELECT_STRATIFIED) {
        passes = K;
        for (int c = lane; c < K; c += kWave) n_in_phase[c] = 0;
        __builtin_amdgcn_wave_barrier();
        for (int k = lane; k < Ni; k += kWave) atomicAdd(&n_in_phase[phase_of(k)], 1);
        __builtin_amdgcn_wave_barrier();
        const int c = lane;                       // K <= 64
        const long long n_c = c < K ? n_in_phase[c] : 0;
        const long long weight = c < K ? n_c * (long long)qtab[c] : 0;
        long long D = weight;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) D += __shfl_xor(D, off, kWave);
        long long b = 0, rem = -1;
        if (c < K && D > 0) {
            b = ((long long)m * weight) / D;
            rem = ((long long)m * weight) % D;
            b = b < n_c ? b : n_c;
        }
        // rank of this phase in the order (larger remainder first, lower index first)
        int rank = 0;
        for (int o = 0; o < K; ++o) {
            const long long ro = __shfl(rem, o, kWave);
            rank += (c < K && (ro > rem || (ro == rem && o < c))) ? 1 : 0;
        }
        long long given = b;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) given += __shfl_xor(given, off, kWave);
        int left = m - (int)given;
        while (left > 0) {                        // each trip serves every phase with room once, in rank order
            const bool room = c < K && b < n_c;
            // position of this phase among those with room, in rank order
            int* has_room = budget;               // indexed by rank
            for (int o = lane; o < K; o += kWave) has_room[o] = 0;
            __builtin_amdgcn_wave_barrier();
            if (room) has_room[rank] = 1;
            __builtin_amdgcn_wave_barrier();
            int before = 0, total = 0;
            for (int o = 0; o < K; ++o) {
                const int h = has_room[o];
                before += (o < rank) ? h : 0;
                total += h;
            }
            __builtin_amdgcn_wave_barrier();
            if (total == 0) break;                // cannot happen: m <= N_i = sum of the caps
            if (room && before < left) b += 1;
            left -= left < total ? left : total;
        }
        __builtin_amdgcn_wave_barrier();
        if (c < K) budget[c] = (int)b;
        __builtin_amdgcn_wave_barrier();
    }

    uint64_t mask = 0;
    uint32_t wreg[kRegs > 0 ? kRegs : 1];     // this lane's weights (kRegs > 0)
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint32_t s0 = (uint32_t)step, s1 = (uint32_t)(step >> 32);
    uint32_t x_lo = 0, x_hi = 0;              // lane l holds the random bits of round (r & ~63) + l
    int r = 0;                                // draw counter, running on across passes
    for (int pass = 0; pass < passes; ++pass) {
        const int draws = selector == PCM_SELECT_STRATIFIED ? budget[pass] : m;
        if (draws == 0) continue;
        uint32_t lane_sum = 0;
        auto weight_of_phase = [&](int k, int c) -> uint32_t {
            if (k >= Ni) return 0u;
            c = c < K ? c : K - 1;
            return selector == PCM_SELECT_STRATIFIED ? (c == pass ? 1u : 0u) : qtab[c];
        };
        auto weight_of = [&](int k) -> uint32_t { return k < Ni ? weight_of_phase(k, ph[k]) : 0u; };
        if (kRegs > 0) {
#pragma unroll
            for (int j = 0; j < kRegs; ++j) {
                wreg[j] = j < per_lane ? weight_of_phase(k_lo + j, my_phase[j]) : 0u;
                lane_sum += wreg[j];
            }
        } else {
            for (int j = 0; j < per_lane; ++j) {
                const int k = k_lo + j;
                const uint32_t wk = weight_of(k);
                if (k < N) w[k] = wk;
                lane_sum += wk;
            }
        }
        uint32_t incl = (uint32_t)wave_inclusive_scan((int)lane_sum, lane);
        uint32_t W_rem = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
        for (int d = 0; d < draws; ++d, ++r) {
            if ((r & (kWave - 1)) == 0) {     // the draws of the next 64 rounds, one per lane, in parallel
                const uint64_t mine = philox_bits((uint32_t)i, (uint32_t)((r & ~(kWave - 1)) + lane), s0, s1, k0, k1);
                x_lo = (uint32_t)mine;
                x_hi = (uint32_t)(mine >> 32);
            }
            const int src = __builtin_amdgcn_readfirstlane(r & (kWave - 1));      // wave-uniform: a lane read, no shuffle
            const uint64_t x = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)x_lo, src) |
                               ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)x_hi, src) << 32);
            const uint32_t t = (uint32_t)__umul64hi(x, (uint64_t)W_rem);   // in [0, W_rem)
            const uint64_t over = __ballot(incl > t);
            if (over == 0) break;             // cannot happen while W_rem > 0; keeps the loop total
            const int L = __ffsll((long long)over) - 1;
            uint32_t picked_w = 0;
            if (lane == L) {
                uint32_t run = incl - lane_sum;
                if (kRegs > 0) {
#pragma unroll
                    for (int j = 0; j < kRegs; ++j) {
                        const uint32_t wk = wreg[j];
                        run += wk;
                        if (picked_w == 0 && wk > 0 && run > t) {   // the first slot whose running weight exceeds t
                            picked_w = wk;
                            wreg[j] = 0;
                            mask |= (uint64_t)1 << j;
                        }
                    }
                } else {
                    for (int j = 0; j < per_lane; ++j) {
                        const int k = k_lo + j;
                        if (k >= N) break;
                        const uint32_t wk = w[k];
                        run += wk;
                        if (wk > 0 && run > t) {
                            picked_w = wk;
                            w[k] = 0;
                            mask |= (uint64_t)1 << j;
                            break;
                        }
                    }
                }
                lane_sum -= picked_w;
            }
            picked_w = (uint32_t)__builtin_amdgcn_readlane((int)picked_w, __builtin_amdgcn_readfirstlane(L));
            if (lane >= L) incl -= picked_w;
            W_rem -= picked_w;
        }
    }

    const int mine = __popcll(mask);
    int pos = offset + wave_inclusive_scan(mine, lane) - mine;
    while (mask) {
        const int j = __ffsll((long long)mask) - 1;
        mask &= mask - 1;
        kept_idx[pos++] = i * N + k_lo + j;
    }
}

bool shape_ok(int T, int N, int K, int B) {
    return T >= 1 && N >= 1 && N <= PCM_MAX_CHUNK_SLOTS && K >= 1 && K <= PCM_MAX_PHASES && B >= 1 &&
           (int64_t)T * N < (int64_t)1 << 31;
}

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" size_t pcm_sample_chunks_workspace_bytes(int T, int N, int K, int B) {
    (void)T; (void)N; (void)K; (void)B;
    return 0;   // offsets and counts live in the caller's output arrays
}

namespace {

int run_sample(const double* keep_probs, const uint8_t* phase, const int32_t* n_chunks, const uint8_t* active, int T,
               int N, int K, int B, int selector, uint64_t seed, uint64_t step, int32_t* kept_idx,
               int32_t* kept_offsets, int32_t* n_kept, void* stream) {
    if (!keep_probs || !phase || !kept_idx || !kept_offsets || !n_kept) return PCM_EINVAL;
    if (!shape_ok(T, N, K, B)) return PCM_EINVAL;
    if (selector != PCM_SELECT_PCM && selector != PCM_SELECT_RANDOM && selector != PCM_SELECT_TOP_PHASE &&
        selector != PCM_SELECT_STRATIFIED)
        return PCM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Every workgroup can find its own output offset from the counts min(B, N_i) of the trajectories before it;
    // beyond kFusedScanMax trajectories that is too much repeated reading, and the top-phase selector's counts
    // need a pass over the phases: then one workgroup scans the counts first.
    const bool fused = T <= kFusedScanMax && selector != PCM_SELECT_TOP_PHASE;
    if (!fused) {
        StageTimer t(ST_SAMPLE_SCAN, s);
        sample_scan<<<1, kThreads, 0, s>>>(keep_probs, phase, n_chunks, active, T, N, K, B, selector, kept_offsets,
                                           n_kept);
    }
    {
        StageTimer t(ST_SAMPLE_COMPACT, s);
        // one weight array per wavefront must fit the 64 KB a workgroup may take by default
        const int waves = N > 2048 ? 2 : kWavesPerBlock;
        const size_t lds_bytes = (PCM_MAX_PHASES + (size_t)waves * (N + 2 * PCM_MAX_PHASES)) * sizeof(uint32_t);
        const int per_lane = ceil_div(N, kWave);
        const dim3 grid(ceil_div(T, waves)), block(waves * kWave);
#define PCM_SAMPLE(REGS, FUSED)                                                                                       \
    sample_compact<REGS, FUSED><<<grid, block, lds_bytes, s>>>(keep_probs, phase, n_chunks, active, T, N, K, B, selector, \
                                                              seed, step, kept_offsets, n_kept, kept_idx)
        if (fused) {
            if (per_lane <= 2) PCM_SAMPLE(2, true);
            else if (per_lane <= 4) PCM_SAMPLE(4, true);
            else if (per_lane <= 8) PCM_SAMPLE(8, true);
            else PCM_SAMPLE(0, true);
        } else {
            if (per_lane <= 4) PCM_SAMPLE(4, false);
            else PCM_SAMPLE(0, false);
        }
#undef PCM_SAMPLE
    }
    return launch_status();
}

// One wavefront per trajectory: per-phase counts of its valid chunks and of its kept chunks in LDS,
// then weight = N_c / b_c for each kept chunk.
__global__ __launch_bounds__(kThreads) void importance_weights(const uint8_t* __restrict__ phase,
                                                               const int32_t* __restrict__ n_chunks,
                                                               const int32_t* __restrict__ kept_idx,
                                                               const int32_t* __restrict__ kept_offsets, int T, int N,
                                                               int K, float* __restrict__ weights) {
    __shared__ int counts[kWavesPerBlock][2][PCM_MAX_PHASES];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int i = blockIdx.x * kWavesPerBlock + wv;
    if (i >= T) return;                       // no workgroup barrier below
    int* all = counts[wv][0];
    int* kept = counts[wv][1];
    for (int c = lane; c < K; c += kWave) {
        all[c] = 0;
        kept[c] = 0;
    }
    __builtin_amdgcn_wave_barrier();
    int Ni = n_chunks ? n_chunks[i] : N;
    Ni = Ni < 0 ? 0 : (Ni > N ? N : Ni);
    const uint8_t* ph = phase + (size_t)i * N;
    for (int k = lane; k < Ni; k += kWave) {
        int c = ph[k];
        c = c < K ? c : K - 1;
        atomicAdd(&all[c], 1);
    }
    const int lo = kept_offsets[i], hi = kept_offsets[i + 1];
    for (int j = lo + lane; j < hi; j += kWave) {
        const int k = kept_idx[j] - i * N;
        int c = (k >= 0 && k < N) ? ph[k] : 0;
        c = c < K ? c : K - 1;
        atomicAdd(&kept[c], 1);
    }
    __builtin_amdgcn_wave_barrier();
    for (int j = lo + lane; j < hi; j += kWave) {
        const int k = kept_idx[j] - i * N;
        int c = (k >= 0 && k < N) ? ph[k] : 0;
        c = c < K ? c : K - 1;
        weights[j] = (float)all[c] / (float)kept[c];
    }
}

// One workgroup: histograms in LDS of the kept chunks' phases and of the phases of all chunk slots the sampler
// could have kept, written out as they are (nothing to clear, no atomics in memory).
__global__ __launch_bounds__(1024) void kept_phase_counts(const uint8_t* __restrict__ phase,
                                                          const int32_t* __restrict__ n_chunks,
                                                          const uint8_t* __restrict__ active,
                                                          const int32_t* __restrict__ kept_idx,
                                                          const int32_t* __restrict__ n_kept, int max_kept, int T, int N,
                                                          int K, int32_t* kept_out, int32_t* eligible_out) {
    __shared__ int hist[2][PCM_MAX_PHASES];
    const int tid = threadIdx.x;
    if (tid < 2 * PCM_MAX_PHASES) hist[tid / PCM_MAX_PHASES][tid % PCM_MAX_PHASES] = 0;
    __syncthreads();
    int nk = *n_kept;
    nk = nk < 0 ? 0 : (nk > max_kept ? max_kept : nk);
    const int64_t slots = (int64_t)T * N;
    for (int j = tid; j < nk; j += 1024) {
        const int id = kept_idx[j];
        if (id >= 0 && id < slots) {
            const int c = phase[id];
            atomicAdd(&hist[0][c < K ? c : K - 1], 1);
        }
    }
    if (eligible_out) {
        for (int64_t e = tid; e < slots; e += 1024) {
            const int i = (int)(e / N), k = (int)(e % N);
            int Ni = n_chunks ? n_chunks[i] : N;
            Ni = Ni > N ? N : Ni;
            if (k < Ni && (!active || active[i])) {
                const int c = phase[e];
                atomicAdd(&hist[1][c < K ? c : K - 1], 1);
            }
        }
    }
    __syncthreads();
    if (tid < K) {
        kept_out[tid] = hist[0][tid];
        if (eligible_out) eligible_out[tid] = hist[1][tid];
    }
}

}  // namespace

extern "C" int pcm_kept_phase_counts(const uint8_t* phase, const int32_t* n_chunks, const uint8_t* active,
                                     const int32_t* kept_idx, const int32_t* n_kept, int max_kept_chunks, int T, int N,
                                     int K, int32_t* kept_per_phase, int32_t* chunks_per_phase, void* stream) {
    if (!phase || !kept_idx || !n_kept || !kept_per_phase || max_kept_chunks < 0) return PCM_EINVAL;
    if (!shape_ok(T, N, K, 1)) return PCM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StageTimer t(ST_SAMPLE_COMPACT, s);
    kept_phase_counts<<<1, 1024, 0, s>>>(phase, n_chunks, active, kept_idx, n_kept, max_kept_chunks, T, N, K, kept_per_phase,
                                         chunks_per_phase);
    return launch_status();
}

extern "C" int pcm_sample_chunks(const double* keep_probs, const uint8_t* phase, const int32_t* n_chunks,
                                 const uint8_t* active, int T, int N, int K, int B, uint64_t seed,
                                 uint64_t step, int32_t* kept_idx, int32_t* kept_offsets, int32_t* n_kept,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    return run_sample(keep_probs, phase, n_chunks, active, T, N, K, B, PCM_SELECT_PCM, seed, step, kept_idx,
                      kept_offsets, n_kept, stream);
}

extern "C" int pcm_sample_chunks_ex(const double* keep_probs, const uint8_t* phase, const int32_t* n_chunks,
                                    const uint8_t* active, int T, int N, int K, int B, int selector, uint64_t seed,
                                    uint64_t step, int32_t* kept_idx, int32_t* kept_offsets, int32_t* n_kept,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    return run_sample(keep_probs, phase, n_chunks, active, T, N, K, B, selector, seed, step, kept_idx, kept_offsets,
                      n_kept, stream);
}

extern "C" int pcm_importance_weights(const uint8_t* phase, const int32_t* n_chunks, const int32_t* kept_idx,
                                      const int32_t* kept_offsets, int T, int N, int K, float* weights, void* stream) {
    if (!phase || !kept_idx || !kept_offsets || !weights) return PCM_EINVAL;
    if (!shape_ok(T, N, K, 1)) return PCM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StageTimer t(ST_SAMPLE_COMPACT, s);
    importance_weights<<<ceil_div(T, kWavesPerBlock), kThreads, 0, s>>>(phase, n_chunks, kept_idx, kept_offsets, T, N,
                                                                        K, weights);
    return launch_status();
}
