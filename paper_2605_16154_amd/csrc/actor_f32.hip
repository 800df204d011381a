// fp32 path of the masked GRPO actor step (Eq. 11): plain vector-ALU kernels.
//
// This path exists for small heads and for checking the method at fp32 accuracy; it is bound by
// the fp32 vector ALUs, not by the matrix cores.  One LDS-tiled GEMM kernel with general strides
// serves all nine products of the forward and backward pass; reductions over the row dimension
// (the weight gradients) are split across workgroups into partial products that a second kernel
// adds in slice order, so the results are the same from run to run (no atomics).
#include <algorithm>

#include "actor.h"

namespace pcm {
namespace {

constexpr int kThreads = 256;
constexpr int BM = 64, BN = 64, BK = 16;

// C[m,n] (+)= sum_k A[m*sam + k*sak] * B[k*sbk + n*sbn]; grid = (tiles_n, tiles_m, splits).
// splits > 1: z-slice q stores its partial product at C + q * split_stride (the caller sums the slices).
__global__ __launch_bounds__(kThreads) void sgemm(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                  const float* __restrict__ B, int64_t sbk, int64_t sbn,
                                                  float* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                  int k_per_split, int accumulate, int64_t split_stride) {
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kb = blockIdx.z * k_per_split;
    const int ke = min(K, kb + k_per_split);
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4] = {};
    for (int k0 = kb; k0 < ke; k0 += BK) {
#pragma unroll
        for (int q = 0; q < (BM * BK) / kThreads; ++q) {
            const int e = tid + q * kThreads;
            int mm, kk;
            if (sak == 1) { mm = e / BK; kk = e % BK; } else { kk = e / BM; mm = e % BM; }
            const int gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < M && gk < ke) ? A[gm * sam + gk * sak] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < (BN * BK) / kThreads; ++q) {
            const int e = tid + q * kThreads;
            int nn, kk;
            if (sbk == 1) { nn = e / BK; kk = e % BK; } else { kk = e / BN; nn = e % BN; }
            const int gn = n0 + nn, gk = k0 + kk;
            Bs[kk][nn] = (gn < N && gk < ke) ? B[gk * sbk + gn * sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][tm + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tn + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + tm + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tn + j;
            if (gn >= N) continue;
            float* c = C + (int64_t)blockIdx.z * split_stride + gm * ldc + gn;
            if (accumulate) *c += acc[i][j];
            else *c = acc[i][j];
        }
    }
}

// out[i] = parts[0][i] + parts[1][i] + ... in slice order (parts are n floats apart).
__global__ void sum_slices(const float* __restrict__ parts, int n_parts, size_t n, float* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float acc = parts[i];
        for (int q = 1; q < n_parts; ++q) acc += parts[(size_t)q * n + i];
        out[i] = acc;
    }
}

__global__ void swiglu_forward(const float* __restrict__ u, const float* __restrict__ v, float* __restrict__ a,
                               size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float x = u[i];
        a[i] = x / (1.f + expf(-x)) * v[i];
    }
}

// In place: u <- du = da * v * silu'(u), v <- dv = da * silu(u).
__global__ void swiglu_backward(float* __restrict__ u, float* __restrict__ v, const float* __restrict__ da,
                                size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float x = u[i], g = da[i], vv = v[i];
        const float s = 1.f / (1.f + expf(-x));
        u[i] = g * vv * (s * (1.f + x * (1.f - s)));
        v[i] = g * (x * s);
    }
}

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) x = fmaxf(x, __shfl_xor(x, d, kWave));
    return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) x += __shfl_xor(x, d, kWave);
    return x;
}

// One wavefront per row: log-softmax at the target bin, entropy, ratio, clipped surrogate, and (in
// place) z <- dz = coef * (onehot - softmax) + entropy part.  With a per-chunk ratio the factor is
// not known yet: z <- onehot - softmax and the entropy part goes to `extra`; the rows are scaled
// once the chunk ratios are known.
__global__ __launch_bounds__(kThreads) void loss_rows(float* __restrict__ z, float* __restrict__ extra, int V,
                                                      const uint8_t* __restrict__ token,
                                                      const float* __restrict__ logp_old,
                                                      const float* __restrict__ adv_row,
                                                      const int32_t* __restrict__ n_kept, int max_chunks, int A,
                                                      int64_t rows_total, LossOptions opt, int write_dz,
                                                      float* logp_out, RowOut out) {
    const int lane = threadIdx.x % kWave;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    if (r >= rows_total) return;
    const int64_t rows = live_rows(n_kept, max_chunks, A);
    const bool live = r < rows;
    const float scale = objective_scale(opt, rows);
    float* zr = z + r * V;
    float mx = -INFINITY;
    for (int j = lane; j < V; j += kWave) mx = fmaxf(mx, zr[j]);
    mx = wave_max(mx);
    float se = 0.f, sz = 0.f;
    for (int j = lane; j < V; j += kWave) {
        const float e = expf(zr[j] - mx);
        se += e;
        sz += e * zr[j];
    }
    se = wave_sum(se);
    sz = wave_sum(sz);
    const int b = token[r];
    const float lse = mx + logf(se);
    const float lp = zr[b] - lse;
    const float H = lse - sz / se;                      // -sum p log p
    const float w = (opt.chunk_weight && live) ? opt.chunk_weight[r / A] : 1.f;
    const LossRow lr = loss_row(lp, logp_old[r], adv_row[r], w, opt, scale);
    if (lane == 0) {
        out.dlogp[r] = lr.dlogp;
        out.entropy[r] = live ? H : 0.f;
        if (!opt.chunk_ratio) {
            out.term[r] = live ? lr.term : 0.f;
            out.ratio[r] = lr.ratio;
            out.clipped[r] = lr.clipped;
        }
        if (logp_out && live) logp_out[r] = lp;
    }
    if (write_dz) {
        const float coef = opt.chunk_ratio ? (live ? 1.f : 0.f) : (live ? lr.coef : 0.f);
        const float ec = live ? opt.entropy_coef * scale : 0.f;
        for (int j = lane; j < V; j += kWave) {
            const float zj = zr[j];
            const float p = expf(zj - lse);
            const float pg = coef * ((j == b ? 1.f : 0.f) - p);
            const float ent = ec * p * (zj - lse + H);
            if (opt.chunk_ratio) {
                zr[j] = pg;
                extra[r * V + j] = ent;
            } else {
                zr[j] = pg + ent;
            }
        }
    }
}

// Reduction split of a product with a small output and a long reduction: enough slices to fill the
// chip, at least four 16-wide steps each.  Returns the slice length; `splits` the number of slices.
int split_of(int M, int N, int K, int& splits) {
    const int tiles = ceil_div(M, BM) * ceil_div(N, BN);
    splits = ceil_div(1024, tiles);
    const int max_splits = ceil_div(K, 4 * BK);
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    const int k_per = ceil_div(ceil_div(K, splits), BK) * BK;
    splits = ceil_div(K, k_per);
    return k_per;
}
size_t split_floats(int M, int N, int K) {
    int splits;
    split_of(M, N, K, splits);
    return splits > 1 ? (size_t)splits * M * N : 0;
}

struct F32Workspace {
    float *X, *u, *v, *a, *y, *z, *z_extra, *dy, *da;
    float *Wdo, *G;   // composed evaluation: Wd Wo and a^T dz, both [ff, V]
    float* parts;     // partial products of the split reductions
    RowMeta meta;
    RowOut out;
    size_t bytes;
};

F32Workspace carve(void* ws, const ActorShape& sh, bool grads) {
    Carver c(ws);
    F32Workspace w{};
    const size_t M = (size_t)sh.rows_max();
    w.X = c.take<float>(M * sh.d);
    w.u = c.take<float>(M * sh.ff);
    w.v = c.take<float>(M * sh.ff);
    w.a = c.take<float>(M * sh.ff);
    w.y = c.take<float>(M * sh.d);
    w.z = c.take<float>(M * sh.V);
    w.meta.token = c.take<uint8_t>(M);
    w.meta.logp_old = c.take<float>(M);
    w.meta.adv = c.take<float>(M);
    w.out.term = c.take<float>(M);
    w.out.ratio = c.take<float>(M);
    w.out.dlogp = c.take<float>(M);
    w.out.clipped = c.take<uint8_t>(M);
    w.out.entropy = c.take<float>(M);
    w.out.coef = c.take<float>(M);
    w.Wdo = c.take<float>((size_t)sh.ff * sh.V);
    w.G = c.take<float>((size_t)sh.ff * sh.V);
    if (grads) {
        w.z_extra = c.take<float>(M * sh.V);
        w.dy = c.take<float>(M * sh.d);
        w.da = c.take<float>(M * sh.ff);
        const int rows = (int)M;
        size_t parts = split_floats(sh.d, sh.V, rows);                       // dWo = y^T dz
        parts = std::max(parts, split_floats(sh.ff, sh.d, rows));             // dWd = a^T dy
        parts = std::max(parts, split_floats(sh.d, sh.ff, rows));             // dWg, dWu
        parts = std::max(parts, split_floats(sh.ff, sh.V, rows));             // composed: G = a^T dz
        parts = std::max(parts, split_floats(sh.d, sh.V, sh.ff));             // composed: dWo = Wd^T G
        w.parts = c.take<float>(parts);
    }
    w.bytes = c.used();
    return w;
}

// C[M,N] (+)= op(A) op(B) with A given as [M,K] row-major (or [K,M] if a_t) and B as [K,N]
// row-major (or [N,K] if b_t).
void gemm(hipStream_t s, const float* A, bool a_t, const float* B, bool b_t, float* C, int M, int N, int K,
          bool accumulate) {
    const int64_t sam = a_t ? 1 : K, sak = a_t ? M : 1;
    const int64_t sbk = b_t ? 1 : N, sbn = b_t ? K : 1;
    dim3 grid(ceil_div(N, BN), ceil_div(M, BM), 1);
    sgemm<<<grid, kThreads, 0, s>>>(A, sam, sak, B, sbk, sbn, C, N, M, N, K, ceil_div(K, BK) * BK, accumulate ? 1 : 0, 0);
}

// C[M,N] = A^T B with A [K,M], B [K,N] row-major: the weight-gradient shape (reduction over rows).
void gemm_reduce_rows(hipStream_t s, const float* A, const float* B, float* C, int M, int N, int K, float* parts) {
    int splits;
    const int k_per = split_of(M, N, K, splits);
    dim3 grid(ceil_div(N, BN), ceil_div(M, BM), splits);
    const size_t n = (size_t)M * N;
    float* dst = splits > 1 ? parts : C;
    sgemm<<<grid, kThreads, 0, s>>>(A, 1, M, B, N, 1, dst, N, M, N, K, k_per, 0, (int64_t)n);
    if (splits > 1) {
        const unsigned blocks = (unsigned)((n + 255) / 256);
        sum_slices<<<blocks < 4096 ? blocks : 4096, 256, 0, s>>>(parts, splits, n, C);
    }
}

}  // namespace

size_t actor_f32_workspace_bytes(const ActorShape& sh, bool want_grads) {
    return carve(nullptr, sh, want_grads).bytes;
}

int actor_f32_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s) {
    const bool bwd = io.want_grads() || io.dX != nullptr;
    F32Workspace w = carve(ws, sh, bwd);
    const int M = (int)sh.rows_max();
    const int d = sh.d, ff = sh.ff, V = sh.V;
    const float* Wg = static_cast<const float*>(io.Wg);
    const float* Wu = static_cast<const float*>(io.Wu);
    const float* Wd = static_cast<const float*>(io.Wd);
    const float* Wo = static_cast<const float*>(io.Wo);
    const size_t n_ff = (size_t)M * ff;
    const unsigned ew_blocks = (unsigned)((n_ff + 1023) / 1024) < 4096 ? (unsigned)((n_ff + 1023) / 1024) : 4096;

    int rc = launch_gather(sh, io, 4, w.X, 0, M, w.meta, s);
    if (rc != PCM_OK) return rc;
    {
        StageTimer t(ST_F32_FORWARD, s);
        gemm(s, w.X, false, Wg, false, w.u, M, ff, d, false);
        gemm(s, w.X, false, Wu, false, w.v, M, ff, d, false);
        swiglu_forward<<<ew_blocks, 256, 0, s>>>(w.u, w.v, w.a, n_ff);
        if (io.composed) {
            gemm(s, Wd, false, Wo, false, w.Wdo, ff, V, d, false);                           // W_do = Wd Wo
            gemm(s, w.a, false, w.Wdo, false, w.z, M, V, ff, false);                         // z = a W_do
        } else {
            gemm(s, w.a, false, Wd, false, w.y, M, d, ff, false);
            gemm(s, w.y, false, Wo, false, w.z, M, V, d, false);
        }
    }
    {
        StageTimer t(ST_F32_LOSS, s);
        loss_rows<<<(unsigned)ceil_div64(M, kThreads / kWave), kThreads, 0, s>>>(
            w.z, w.z_extra, V, w.meta.token, w.meta.logp_old, w.meta.adv, io.n_kept, sh.max_chunks, sh.A, M, io.opt,
            bwd ? 1 : 0, io.logp_out, w.out);
    }
    if (io.opt.chunk_ratio) {
        rc = launch_chunk_ratio(sh, io, w.meta, w.out, 0, M, s);
        if (rc != PCM_OK) return rc;
        if (bwd) {
            rc = launch_scale_rows(sh, io, w.z, io.opt.entropy_coef != 0.f ? w.z_extra : nullptr, w.out.coef, 0, M, 4, s);
            if (rc != PCM_OK) return rc;
        }
    }
    rc = launch_loss_reduce(sh, io, w.out, SumsqLists{}, s);
    if (rc != PCM_OK) return rc;
    if (!bwd) return launch_status();
    {
        StageTimer t(ST_F32_BACKWARD, s);
        float* dz = w.z;
        if (io.want_grads()) {
            if (io.composed) {
                gemm_reduce_rows(s, w.a, dz, w.G, ff, V, M, w.parts);                           // G = a^T dz
                gemm(s, w.G, false, Wo, true, io.dWd, ff, d, V, false);                         // dWd = G Wo^T
                gemm_reduce_rows(s, Wd, w.G, io.dWo, d, V, ff, w.parts);                        // dWo = Wd^T G
            } else {
                gemm_reduce_rows(s, w.y, dz, io.dWo, d, V, M, w.parts);                         // dWo = y^T dz
            }
        }
        if (io.composed) {
            gemm(s, dz, false, w.Wdo, true, w.da, M, ff, V, false);                             // da = dz W_do^T
        } else {
            gemm(s, dz, false, Wo, true, w.dy, M, d, V, false);                                 // dy = dz Wo^T
            if (io.want_grads()) gemm_reduce_rows(s, w.a, w.dy, io.dWd, ff, d, M, w.parts);     // dWd = a^T dy
            gemm(s, w.dy, false, Wd, true, w.da, M, ff, d, false);                              // da = dy Wd^T
        }
        swiglu_backward<<<ew_blocks, 256, 0, s>>>(w.u, w.v, w.da, n_ff);                        // u <- du, v <- dv
        if (io.want_grads()) {
            gemm_reduce_rows(s, w.X, w.u, io.dWg, d, ff, M, w.parts);                           // dWg = X^T du
            gemm_reduce_rows(s, w.X, w.v, io.dWu, d, ff, M, w.parts);                           // dWu = X^T dv
        }
        if (io.dX) {
            float* dX = static_cast<float*>(io.dX);
            gemm(s, w.u, false, Wg, true, dX, M, d, ff, false);                              // dX = du Wg^T
            gemm(s, w.v, false, Wu, true, dX, M, d, ff, true);                               //    + dv Wu^T
        }
    }
    return launch_status();
}

}  // namespace pcm
