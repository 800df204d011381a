// Physical shrinking of the batch (Sec. 4.5): copy the kept chunks' hidden rows into a dense
// matrix and expand the per-trajectory advantage to rows; plus the fixed-order reduction of the
// per-row loss terms of Eq. 11.
//
// The gather is a pure streaming copy (row r of the compacted batch is token r % A of chunk
// kept_idx[r / A]); each workgroup moves a block of rows with 16-byte accesses, several loads in
// flight per lane.  Rows at and beyond n_kept * A are zero-filled with advantage 0, so they add
// nothing downstream.
#include "actor.h"

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = 8;

template <typename Vec>
__device__ inline Vec zero_vec();
template <>
__device__ inline uint4 zero_vec<uint4>() { return make_uint4(0, 0, 0, 0); }
template <>
__device__ inline uint32_t zero_vec<uint32_t>() { return 0u; }
template <>
__device__ inline uint16_t zero_vec<uint16_t>() { return 0; }

template <typename Vec>
__global__ __launch_bounds__(kThreads) void gather_rows(
    const Vec* __restrict__ hidden, const uint8_t* __restrict__ tokens, const float* __restrict__ logp_old,
    const float* __restrict__ adv, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ n_kept,
    int max_chunks, int T, int N, int A, int V, int vec_per_row, int64_t row_offset, int64_t rows_pad,
    Vec* __restrict__ X, uint8_t* m_token, float* m_logp_old, float* m_adv) {
    // rows are those of a panel that starts at batch row row_offset; X and the m_ arrays are the panel's
    __shared__ int64_t src_row[kRowsPerBlock];
    int nk = *n_kept;
    nk = nk < 0 ? 0 : (nk > max_chunks ? max_chunks : nk);
    const int64_t rows_valid = (int64_t)nk * A - row_offset;
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlock;
    const int tid = threadIdx.x;
    if (tid < kRowsPerBlock) {
        const int64_t r = r0 + tid;
        int64_t src = -1;
        if (r < rows_valid) {
            const int ci = (int)((r + row_offset) / A), tok = (int)((r + row_offset) % A);
            int id = kept_idx[ci];
            float a = 0.f;
            if (id >= 0 && (int64_t)id < (int64_t)T * N) a = adv[id / N];
            else id = 0;
            src = (int64_t)id * A + tok;
            int b = tokens[src];
            m_token[r] = (uint8_t)(b < V ? b : V - 1);
            m_logp_old[r] = logp_old[src];
            m_adv[r] = a;
        } else if (r < rows_pad) {
            m_token[r] = 0;
            m_logp_old[r] = 0.f;
            m_adv[r] = 0.f;
        }
        src_row[tid] = src;
    }
    __syncthreads();
    const int total = kRowsPerBlock * vec_per_row;
    constexpr int kUnroll = 8;
    for (int base = tid; base < total; base += kThreads * kUnroll) {
        Vec v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int e = base + u * kThreads;
            v[u] = zero_vec<Vec>();
            if (e < total) {
                const int64_t src = src_row[e / vec_per_row];
                if (src >= 0) v[u] = hidden[src * vec_per_row + e % vec_per_row];
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int e = base + u * kThreads;
            if (e < total) {
                const int64_t r = r0 + e / vec_per_row;
                if (r < rows_pad) X[r * vec_per_row + e % vec_per_row] = v[u];
            }
        }
    }
}

// One workgroup; lane-strided fp64 partials combined by a fixed tree, so the result does not
// depend on anything but the row values.
__global__ __launch_bounds__(1024) void loss_reduce(const float* __restrict__ term,
                                                     const float* __restrict__ ratio,
                                                     const float* __restrict__ dlogp,
                                                     const uint8_t* __restrict__ clipped,
                                                     const float* __restrict__ entropy,
                                                     const int32_t* __restrict__ n_kept, int max_chunks, int A,
                                                     LossOptions opt, float* loss_out, float* stats_out, int n_stats,
                                                     SumsqLists lists) {
    __shared__ double red[5][1024];
    const int64_t rows = live_rows(n_kept, max_chunks, A);
    double acc[5] = {0, 0, 0, 0, 0};
    for (int64_t r = threadIdx.x; r < rows; r += 1024) {
        acc[0] += (double)term[r];
        acc[1] += (double)ratio[r];
        acc[2] += (double)dlogp[r];
        acc[3] += (double)clipped[r];
        acc[4] += (double)entropy[r];
    }
    for (int q = 0; q < 5; ++q) red[q][threadIdx.x] = acc[q];
    __syncthreads();
    for (int half = 512; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half)
            for (int q = 0; q < 5; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + half];
        __syncthreads();
    }
    if (opt.grad_sumsq_out != nullptr && lists.parts[0] != nullptr) {   // uniform over the workgroup
        __shared__ double red_sq[1024];
        double sq = 0.0;
        for (int q = 0; q < 4; ++q)
            for (int i = threadIdx.x; i < lists.count[q]; i += 1024) sq += lists.parts[q][i];
        red_sq[threadIdx.x] = sq;
        __syncthreads();
        for (int half = 512; half > 0; half >>= 1) {
            if ((int)threadIdx.x < half) red_sq[threadIdx.x] += red_sq[threadIdx.x + half];
            __syncthreads();
        }
        if (threadIdx.x == 0) *opt.grad_sumsq_out = red_sq[0];
    }
    if (threadIdx.x == 0) {
        const double scale = (double)objective_scale(opt, rows);
        *loss_out = (float)(-scale * red[0][0] - (double)opt.entropy_coef * scale * red[4][0]);
        if (stats_out) {
            const double n = rows > 0 ? (double)rows : 1.0;
            stats_out[0] = (float)(red[3][0] / n);
            stats_out[1] = (float)(red[1][0] / n);
            stats_out[2] = (float)(red[2][0] / n);
            stats_out[3] = (float)rows;
            if (n_stats > 4) stats_out[4] = (float)(red[4][0] / n);
        }
    }
}

// One lane per chunk slot.  rho_c = exp(sum over the chunk's tokens of (logp - logp_old)).
__global__ __launch_bounds__(256) void chunk_ratio_rows(const float* __restrict__ dlogp,
                                                        const float* __restrict__ adv_row,
                                                        const int32_t* __restrict__ n_kept, int max_chunks, int A,
                                                        int64_t row_offset, int64_t rows_pad, LossOptions opt,
                                                        float* __restrict__ term, float* __restrict__ ratio,
                                                        uint8_t* __restrict__ clipped, float* __restrict__ coef) {
    // chunk slots of a panel that starts at batch row row_offset (a multiple of A); the arrays are the panel's
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r0 = c * A;
    if (r0 >= rows_pad) return;
    const int64_t rows_batch = live_rows(n_kept, max_chunks, A);
    const int64_t rows = rows_batch - row_offset;
    const int64_t r1 = r0 + A < rows_pad ? r0 + A : rows_pad;
    if (r0 >= rows) return;                             // beyond the kept chunks: nothing reads these rows
    float sum = 0.f;
    for (int64_t r = r0; r < r1; ++r) sum -= dlogp[r];
    const float w = opt.chunk_weight ? opt.chunk_weight[c + row_offset / A] : 1.f;
    const LossRow lr = loss_from_ratio(expf(sum), adv_row[r0], w, opt, objective_scale(opt, rows_batch));
    for (int64_t r = r0; r < r1; ++r) {
        term[r] = r == r0 ? lr.term : 0.f;
        ratio[r] = lr.ratio;
        clipped[r] = lr.clipped;
        coef[r] = lr.coef;
    }
}

template <typename T>
__device__ inline float to_f32(T x);
template <>
__device__ inline float to_f32<float>(float x) { return x; }
template <>
__device__ inline float to_f32<bf16>(bf16 x) { return __bfloat162float(x); }
template <typename T>
__device__ inline T from_f32(float x);
template <>
__device__ inline float from_f32<float>(float x) { return x; }
template <>
__device__ inline bf16 from_f32<bf16>(float x) { return __float2bfloat16(x); }

// Rows [0, live rows) only: rows beyond them hold zeros (or, in row tiles that the logit product
// skipped, nothing) and are not read by anything downstream.
template <typename T>
__global__ __launch_bounds__(256) void scale_rows(T* __restrict__ dz, const T* __restrict__ extra,
                                                   const float* __restrict__ coef, const int32_t* __restrict__ n_kept,
                                                   int max_chunks, int A, int64_t row_offset, int64_t rows_pad, int V) {
    int64_t rows = live_rows(n_kept, max_chunks, A) - row_offset;
    rows = rows < rows_pad ? rows : rows_pad;
    const int64_t n = rows * V;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float x = coef[i / V] * to_f32<T>(dz[i]);
        if (extra) x += to_f32<T>(extra[i]);
        dz[i] = from_f32<T>(x);
    }
}

// Whether panel row r (batch row r + row_offset) carries a gradient.
struct RowGradient {
    const uint8_t* clipped;
    const float* adv;
    const float* chunk_weight;   // by chunk of the batch, or null
    int64_t row_offset;
    int A;
    __device__ bool operator()(int r) const {      // all loads unconditional, so that a loop of calls can overlap them
        const uint8_t cut = clipped[r];
        const float a = adv[r];
        const float w = chunk_weight != nullptr ? chunk_weight[(r + row_offset) / A] : 1.f;
        return cut == 0 && a != 0.f && w != 0.f;
    }
};

// Rows whose gradient factor is zero (ratio cut by the clip, zero advantage, zero weight) have an all-zero row of
// dz and add nothing to any gradient.  One workgroup lists the panel's rows with a non-zero factor, in order, and
// decides whether the backward products run over that list or over all live rows.
// Rows are swept 1024 at a time (thread t looks at row 1024 q + t, so reads are contiguous); a sweep of kListRounds
// such rounds first counts the rows with a gradient per round and wavefront, turns the counts into positions with
// one scan, then writes the row numbers.
constexpr int kListRounds = 64;   // one bit each in a 64-bit word per thread
__global__ __launch_bounds__(1024) void live_row_list(RowGradient has_gradient, const int32_t* __restrict__ n_kept,
                                                       int max_chunks, int A, int64_t row_offset, int rows_pad,
                                                       LiveSources whole, LiveSources listed, int32_t* __restrict__ idx,
                                                       LivePlan* __restrict__ plan) {
    __shared__ int32_t count[kListRounds * 16];   // [round][wavefront], then the position of its first listed row
    __shared__ int32_t wave_sum[16];
    int64_t rows64 = live_rows(n_kept, max_chunks, A) - row_offset;
    const int rows = (int)(rows64 < 0 ? 0 : (rows64 > rows_pad ? rows_pad : rows64));
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int total = 0;
    for (int sweep0 = 0; sweep0 < rows; sweep0 += kListRounds * 1024) {
        // this thread's rows of the sweep, one bit per round; read first (independent loads, many in flight), the
        // wavefront votes afterwards
        uint64_t mine_bits = 0;
#pragma unroll 8
        for (int q = 0; q < kListRounds; ++q) {
            const int r = sweep0 + q * 1024 + t;
            const bool g = has_gradient(r < rows ? r : rows - 1);
            if (r < rows && g) mine_bits |= 1ull << q;
        }
        for (int q = 0; q < kListRounds; ++q) {
            const uint64_t mask = __ballot((mine_bits >> q) & 1ull);
            if (lane == 0) count[q * 16 + wave] = __popcll(mask);
        }
        __syncthreads();
        const int mine = count[t];                       // entry t = (round t / 16, wavefront t % 16): row order
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int before = 0, sweep_total = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int v = wave_sum[q];
            before += q < wave ? v : 0;
            sweep_total += v;
        }
        count[t] = total + before + incl - mine;
        __syncthreads();
        for (int q = 0; q < kListRounds; ++q) {
            const bool live = (mine_bits >> q) & 1ull;
            const uint64_t mask = __ballot(live);
            if (live) idx[count[q * 16 + wave] + __popcll(mask & ((1ull << lane) - 1ull))] = sweep0 + q * 1024 + t;
        }
        total += sweep_total;
        __syncthreads();
    }
    // the list pays once the rows it drops outweigh the copies it needs: at least one row in sixteen
    const bool use_list = (int64_t)(rows - total) * 16 >= rows && rows > 0;
    const int n = use_list ? total : rows;
    if (!use_list)
        for (int r = t; r < rows; r += 1024) idx[r] = r;
    for (int m = n + t; m < (n + 255) / 256 * 256; m += 1024) idx[m] = -1;   // up to the end of the last row tile
    if (t == 0) {
        plan->n_rows = n;
        plan->listed = use_list ? 1 : 0;
        for (int q = 0; q < LiveSources::kCount; ++q) plan->src[q] = use_list ? listed.p[q] : whole.p[q];
    }
}

// dst[m] = src[idx[m]] for the listed rows, zero rows from there to the end of the last row tile; nothing when
// the backward products run over all live rows.  Rows are row_vecs 16-byte units long; a workgroup moves blocks of
// kRowsPerBlock rows, striding over the blocks by the grid.
__global__ __launch_bounds__(kThreads) void gather_listed_rows(const uint4* __restrict__ src, const int32_t* __restrict__ idx,
                                                               const LivePlan* __restrict__ plan, int row_vecs,
                                                               uint4* __restrict__ dst) {
    __shared__ int32_t src_row[kRowsPerBlock];
    if (!plan->listed) return;
    const int limit = (plan->n_rows + 255) / 256 * 256;
    const int tid = threadIdx.x;
    const int total = kRowsPerBlock * row_vecs;
    constexpr int kUnroll = 8;
    for (int r0 = blockIdx.x * kRowsPerBlock; r0 < limit; r0 += gridDim.x * kRowsPerBlock) {
        __syncthreads();
        if (tid < kRowsPerBlock) src_row[tid] = idx[r0 + tid];
        __syncthreads();
        for (int base = tid; base < total; base += kThreads * kUnroll) {
            uint4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int el = base + u * kThreads;
                v[u] = make_uint4(0, 0, 0, 0);
                if (el < total) {
                    const int row = src_row[el / row_vecs];
                    if (row >= 0) v[u] = src[(int64_t)row * row_vecs + el % row_vecs];
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int el = base + u * kThreads;
                if (el < total) dst[(int64_t)(r0 + el / row_vecs) * row_vecs + el % row_vecs] = v[u];
            }
        }
    }
}

// Zero rows of dX for the panel rows the listed products do not write: rows without a gradient, and the rows
// between the live rows and the end of their row tile (as far as dX has them).
__global__ __launch_bounds__(kThreads) void zero_unlisted_rows(RowGradient has_gradient,
                                                               const int32_t* __restrict__ n_kept, int max_chunks, int A,
                                                               int64_t row_offset, int rows_pad, int rows_in_dX,
                                                               int row_vecs, uint4* __restrict__ dX) {
    int64_t rows64 = live_rows(n_kept, max_chunks, A) - row_offset;
    const int rows = (int)(rows64 < 0 ? 0 : (rows64 > rows_pad ? rows_pad : rows64));
    const int limit = min(rows_in_dX, (rows + 255) / 256 * 256);
    for (int r = blockIdx.x; r < limit; r += gridDim.x) {
        if (r < rows && has_gradient(r)) continue;
        for (int c = threadIdx.x; c < row_vecs; c += kThreads) dX[(int64_t)r * row_vecs + c] = make_uint4(0, 0, 0, 0);
    }
}

}  // namespace

int launch_live_row_list(const ActorShape& sh, const ActorIO& io, const uint8_t* clipped, const float* adv,
                         int64_t row_offset, int64_t rows_pad, const LiveSources& whole, const LiveSources& listed,
                         int32_t* idx, LivePlan* plan, hipStream_t s) {
    const RowGradient g{clipped, adv, io.opt.chunk_weight, row_offset, sh.A};
    live_row_list<<<1, 1024, 0, s>>>(g, io.n_kept, sh.max_chunks, sh.A, row_offset, (int)rows_pad, whole, listed, idx, plan);
    return launch_status();
}

int launch_gather_listed(const void* src, const int32_t* idx, const LivePlan* plan, int64_t rows_pad, int64_t row_bytes,
                         void* dst, hipStream_t s) {
    const int64_t blocks = ceil_div64(rows_pad, kRowsPerBlock);
    gather_listed_rows<<<(unsigned)(blocks < 2048 ? blocks : 2048), kThreads, 0, s>>>(
        static_cast<const uint4*>(src), idx, plan, (int)(row_bytes / 16), static_cast<uint4*>(dst));
    return launch_status();
}

int launch_zero_unlisted(const ActorShape& sh, const ActorIO& io, const uint8_t* clipped, const float* adv,
                         int64_t row_offset, int64_t rows_pad, int64_t rows_in_dX, int64_t row_bytes, void* dX,
                         hipStream_t s) {
    const RowGradient g{clipped, adv, io.opt.chunk_weight, row_offset, sh.A};
    zero_unlisted_rows<<<(unsigned)(rows_pad < 2048 ? rows_pad : 2048), kThreads, 0, s>>>(
        g, io.n_kept, sh.max_chunks, sh.A, row_offset, (int)rows_pad, (int)rows_in_dX, (int)(row_bytes / 16),
        static_cast<uint4*>(dX));
    return launch_status();
}

int launch_gather(const ActorShape& sh, const ActorIO& io, int elem_bytes, void* X, int64_t row_offset, int64_t rows_pad,
                  RowMeta meta, hipStream_t s) {
    StageTimer t(ST_GATHER, s);
    const int64_t row_bytes = (int64_t)sh.d * elem_bytes;
    const unsigned blocks = (unsigned)ceil_div64(rows_pad, kRowsPerBlock);
    const bool aligned16 = row_bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(io.hidden) & 15u) == 0 &&
                           (reinterpret_cast<uintptr_t>(X) & 15u) == 0;
#define PCM_GATHER(Vec, vpr)                                                                             \
    gather_rows<Vec><<<blocks, kThreads, 0, s>>>(static_cast<const Vec*>(io.hidden), io.tokens,          \
                                                 io.logp_old, io.adv, io.kept_idx, io.n_kept,            \
                                                 sh.max_chunks, sh.T, sh.N, sh.A, sh.V, (int)(vpr),      \
                                                 row_offset, rows_pad, static_cast<Vec*>(X), meta.token, \
                                                 meta.logp_old, meta.adv)
    if (aligned16) PCM_GATHER(uint4, row_bytes / 16);
    else if (elem_bytes == 4) PCM_GATHER(uint32_t, sh.d);
    else PCM_GATHER(uint16_t, sh.d);
#undef PCM_GATHER
    return launch_status();
}

int launch_loss_reduce(const ActorShape& sh, const ActorIO& io, RowOut out, const SumsqLists& lists, hipStream_t s) {
    StageTimer t(ST_REDUCE, s);
    loss_reduce<<<1, 1024, 0, s>>>(out.term, out.ratio, out.dlogp, out.clipped, out.entropy, io.n_kept,
                                   sh.max_chunks, sh.A, io.opt, io.loss_out, io.stats_out, io.n_stats, lists);
    return launch_status();
}

int launch_chunk_ratio(const ActorShape& sh, const ActorIO& io, RowMeta meta, RowOut out, int64_t row_offset,
                       int64_t rows_pad, hipStream_t s) {
    StageTimer t(ST_REDUCE, s);
    const int64_t slots = ceil_div64(rows_pad, sh.A);
    chunk_ratio_rows<<<(unsigned)ceil_div64(slots, 256), 256, 0, s>>>(out.dlogp, meta.adv, io.n_kept, sh.max_chunks,
                                                                      sh.A, row_offset, rows_pad, io.opt, out.term,
                                                                      out.ratio, out.clipped, out.coef);
    return launch_status();
}

int launch_scale_rows(const ActorShape& sh, const ActorIO& io, void* dz, const void* extra, const float* coef,
                      int64_t row_offset, int64_t rows_pad, int elem_bytes, hipStream_t s) {
    StageTimer t(ST_REDUCE, s);
    const int64_t n = rows_pad * sh.V;
    unsigned blocks = (unsigned)(ceil_div64(n, 256) < 4096 ? ceil_div64(n, 256) : 4096);
    if (elem_bytes == 2)
        scale_rows<bf16><<<blocks, 256, 0, s>>>(static_cast<bf16*>(dz), static_cast<const bf16*>(extra), coef, io.n_kept,
                                                sh.max_chunks, sh.A, row_offset, rows_pad, sh.V);
    else
        scale_rows<float><<<blocks, 256, 0, s>>>(static_cast<float*>(dz), static_cast<const float*>(extra), coef,
                                                 io.n_kept, sh.max_chunks, sh.A, row_offset, rows_pad, sh.V);
    return launch_status();
}

}  // namespace pcm
