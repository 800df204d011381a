// bf16 matrix-core GEMM for gfx950 with fused epilogues (internal header).
//
// C[m, n] = sum_k A[m, k] * B[n, k]: both operands are stored with the reduction index
// contiguous ("NT"), which is the layout the MFMA operand registers want (each lane feeds 8
// consecutive k of one row).  Products that are not naturally in this form get a transposed copy
// of one operand from a separate streaming kernel.
//
// Tiling: 256 x 256 x 64 per workgroup of 4 wavefronts (2 x 2), each wavefront owning 128 x 128 =
// 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 with fp32 accumulators (256 accumulator registers per
// lane, one wavefront per SIMD).  Operand tiles are double-buffered in LDS (2 x 64 KB) and filled
// by direct global-to-LDS loads (no staging registers); rows are 128 B and the eight 16-byte
// pieces of a row are XOR-swizzled with the row index so that the 16-byte fragment reads spread
// over all banks.
//
// The MFMA is issued with the B fragment as the first operand, so the accumulator tile is the
// transpose of the usual one: a lane holds, for one output row m, runs of 4 consecutive n.
// Epilogues therefore see 4-wide row-contiguous vectors (8-byte bf16 stores).
#pragma once

#include "actor.h"

namespace pcm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kTileM = 256, kTileN = 256, kTileK = 64;
constexpr int kGemmThreads = 256;
constexpr int kNumXcd = 8;

struct GemmProblem {
    const bf16* A;    // [M, K1] row-major, leading dimension lda
    const bf16* B;    // [N, K1] row-major, leading dimension ldb
    const bf16* A2;   // optional second reduction segment (same M, N), K2 columns
    const bf16* B2;
    int64_t lda, ldb, lda2, ldb2;
    int M, N, K1, K2;  // M, N multiples of 256; K1, K2 multiples of 64
    int splits;        // reduction split (grid multiplies by it); epilogue must combine partials
};

// Accumulator coordinates.  For tile (i, j) of the wavefront and register e = 4 * q + t:
//   row  m = m0 + wm * 128 + i * 32 + (lane & 31)
//   col  n = n0 + wn * 128 + j * 32 + 8 * q + 4 * (lane >> 5) + t
struct TileCoord {
    int m0, n0, wm, wn, lane;
    __device__ int row(int i) const { return m0 + wm * 128 + i * 32 + (lane & 31); }
    __device__ int col(int j, int q) const { return n0 + wn * 128 + j * 32 + 8 * q + 4 * (lane >> 5); }
};

__device__ inline bf16x4 to_bf16x4(float a, float b, float c, float d) {
    bf16x4 r;
    r[0] = (__bf16)a; r[1] = (__bf16)b; r[2] = (__bf16)c; r[3] = (__bf16)d;
    return r;
}

__device__ inline int swizzle_piece(int row, int piece) { return piece ^ (row & 7); }

// Workgroup id -> (tile_m, tile_n).  Consecutive hardware workgroup ids go to different XCDs, each
// with its own L2, so ids are first regrouped so that one XCD works on a contiguous range of
// tiles, then tiles are walked in column-major bands of 8 row-tiles to reuse operand panels.
__device__ inline void tile_of_workgroup(int wg, int n_wg, int tiles_m, int tiles_n, int& tm, int& tn) {
    int logical = wg;
    if (n_wg % kNumXcd == 0) logical = (wg % kNumXcd) * (n_wg / kNumXcd) + wg / kNumXcd;
    constexpr int kBand = 8;
    const int band_size = kBand * tiles_n;
    const int band = logical / band_size;
    const int first = band * kBand;
    const int rows = min(tiles_m - first, kBand);
    const int in_band = logical % band_size;
    tm = first + in_band % rows;
    tn = in_band / rows;
}

#define PCM_AS_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PCM_AS_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

template <class Epilogue>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_nt(GemmProblem p, Epilogue epi) {
    // two stages of (A tile, B tile); separate objects so that loads into one stage are known not
    // to alias fragment reads from the other
    __shared__ __attribute__((aligned(1024))) __bf16 sA0[kTileM * kTileK];
    __shared__ __attribute__((aligned(1024))) __bf16 sB0[kTileN * kTileK];
    __shared__ __attribute__((aligned(1024))) __bf16 sA1[kTileM * kTileK];
    __shared__ __attribute__((aligned(1024))) __bf16 sB1[kTileN * kTileK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_m = p.M / kTileM, tiles_n = p.N / kTileN;
    const int n_tiles = tiles_m * tiles_n;
    const int split = blockIdx.x / n_tiles;
    int tm, tn;
    tile_of_workgroup(blockIdx.x % n_tiles, n_tiles, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * kTileM, n0 = tn * kTileN;

    // reduction range of this workgroup, in 64-wide steps over the concatenation of both segments
    const int steps1 = p.K1 / kTileK, steps_all = steps1 + p.K2 / kTileK;
    const int per_split = (steps_all + p.splits - 1) / p.splits;
    const int step_begin = split * per_split;
    const int step_end = min(steps_all, step_begin + per_split);

    // Global -> LDS without passing through registers: one wave-wide load fills 1 KB of LDS (8 tile
    // rows), lane l landing in 16-byte slot l.  The swizzle is therefore applied on the global
    // side: the lane that lands in slot (row, piece') fetches piece' ^ swizzle(row) of that row.
    // Wave w fills rows [64 w, 64 w + 64) of both tiles with 8 loads each.
    const int ld_row = wave * 64 + (lane >> 3);                 // + 8 * r for load r
    const int ld_piece = swizzle_piece(ld_row, lane & 7);       // (row + 8 r) has the same low 3 bits
    auto issue_loads = [&](__bf16* sa, __bf16* sb, int step) {
        const bf16 *a, *b;
        int64_t la, lb;
        int k0;
        if (step < steps1) { a = p.A; b = p.B; la = p.lda; lb = p.ldb; k0 = step * kTileK; }
        else { a = p.A2; b = p.B2; la = p.lda2; lb = p.ldb2; k0 = (step - steps1) * kTileK; }
        const bf16* ap = a + (int64_t)(m0 + ld_row) * la + k0 + ld_piece * 8;
        const bf16* bp = b + (int64_t)(n0 + ld_row) * lb + k0 + ld_piece * 8;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            __builtin_amdgcn_global_load_lds(PCM_AS_GLOBAL(ap + (int64_t)r * 8 * la),
                                             PCM_AS_LDS(sa + (wave * 64 + r * 8) * kTileK), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(PCM_AS_GLOBAL(bp + (int64_t)r * 8 * lb),
                                             PCM_AS_LDS(sb + (wave * 64 + r * 8) * kTileK), 16, 0, 0);
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto compute = [&](const __bf16* sa, const __bf16* sb) {
#pragma unroll
        for (int ks = 0; ks < kTileK / 16; ++ks) {
            bf16x8 fa[4], fb[4];
            const int piece = ks * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = wm * 128 + i * 32 + (lane & 31);
                fa[i] = *reinterpret_cast<const bf16x8*>(sa + row * kTileK + swizzle_piece(row, piece) * 8);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = wn * 128 + j * 32 + (lane & 31);
                fb[j] = *reinterpret_cast<const bf16x8*>(sb + row * kTileK + swizzle_piece(row, piece) * 8);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
    };

    const int n_steps = step_end - step_begin;
    if (n_steps > 0) {
        issue_loads(sA0, sB0, step_begin);
        __syncthreads();
        // two steps per trip so that each stage is a fixed LDS object; a trailing odd step follows
        for (int pair = 0; pair < n_steps / 2; ++pair) {
            const int step = step_begin + 2 * pair;
            issue_loads(sA1, sB1, step + 1);
            compute(sA0, sB0);
            __syncthreads();
            if (step + 2 < step_end) issue_loads(sA0, sB0, step + 2);
            compute(sA1, sB1);
            __syncthreads();
        }
        if (n_steps & 1) compute(sA0, sB0);
        __syncthreads();
    }

    TileCoord tc{m0, n0, wm, wn, lane};
    epi(tc, acc, reinterpret_cast<float*>(sA0));
}

// ---- epilogues -------------------------------------------------------------------------------

// C (bf16, row-major) = acc; rows at and beyond row_limit are not written.
struct EpiStoreBf16 {
    bf16* C;
    int64_t ldc;
    int row_limit;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], float*) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
            if (m >= row_limit) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& a = acc[i][j];
                    *reinterpret_cast<bf16x4*>(C + (int64_t)m * ldc + tc.col(j, q)) =
                        to_bf16x4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]);
                }
        }
    }
};

// C (fp32, row-major) += acc with atomics (partials of a split reduction) or = acc.
struct EpiAccumulateF32 {
    float* C;
    int64_t ldc;
    int atomic;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], float*) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float* c = C + (int64_t)m * ldc + tc.col(j, q);
                    const f32x16& a = acc[i][j];
                    if (atomic) {
#pragma unroll
                        for (int t = 0; t < 4; ++t) atomicAdd(c + t, a[4 * q + t]);
                    } else {
                        f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                        *reinterpret_cast<f32x4*>(c) = v;
                    }
                }
        }
    }
};

// Gate/up projection with the activation fused: the B operand holds, per 128 packed rows, 64 gate
// columns followed by the 64 up columns of the same index range, so a wavefront's tiles j = 0, 1
// are u and j = 2, 3 the matching v.  Writes u, v and a = silu(u) * v (bf16, [M, ff]).
struct EpiSwigluForward {
    bf16 *u, *v, *a;
    int64_t ld;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], float*) const {
        const int col_base = ((tc.n0 + tc.wn * 128) / 128) * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = col_base + j * 32 + 8 * q + 4 * (tc.lane >> 5);
                    float uu[4], vv[4], aa[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        // round u and v first: the backward pass sees the stored values
                        uu[t] = (float)(__bf16)acc[i][j][4 * q + t];
                        vv[t] = (float)(__bf16)acc[i][j + 2][4 * q + t];
                        aa[t] = uu[t] / (1.f + __expf(-uu[t])) * vv[t];
                    }
                    const int64_t off = (int64_t)m * ld + n;
                    *reinterpret_cast<bf16x4*>(u + off) = to_bf16x4(uu[0], uu[1], uu[2], uu[3]);
                    *reinterpret_cast<bf16x4*>(v + off) = to_bf16x4(vv[0], vv[1], vv[2], vv[3]);
                    *reinterpret_cast<bf16x4*>(a + off) = to_bf16x4(aa[0], aa[1], aa[2], aa[3]);
                }
        }
    }
};

// acc = da.  In place: u <- du = da * v * silu'(u), v <- dv = da * silu(u)  (bf16, [M, ff]).
struct EpiSwigluBackward {
    bf16 *u, *v;
    int64_t ld;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], float*) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t off = (int64_t)m * ld + tc.col(j, q);
                    const bf16x4 u4 = *reinterpret_cast<const bf16x4*>(u + off);
                    const bf16x4 v4 = *reinterpret_cast<const bf16x4*>(v + off);
                    float du[4], dv[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float x = (float)u4[t], g = acc[i][j][4 * q + t];
                        const float s = 1.f / (1.f + __expf(-x));
                        du[t] = g * (float)v4[t] * (s * (1.f + x * (1.f - s)));
                        dv[t] = g * (x * s);
                    }
                    *reinterpret_cast<bf16x4*>(u + off) = to_bf16x4(du[0], du[1], du[2], du[3]);
                    *reinterpret_cast<bf16x4*>(v + off) = to_bf16x4(dv[0], dv[1], dv[2], dv[3]);
                }
        }
    }
};

// Logit projection (N = V = 256 = one tile, so a workgroup holds whole rows) with the loss fused:
// log-softmax at the target bin, ratio, clipped surrogate, dz = coef * (onehot - softmax) as bf16.
struct EpiLogitsLoss {
    const uint8_t* token;
    const float* logp_old;
    const float* adv_row;
    const int32_t* n_kept;
    int max_chunks, A;
    float eps_low, eps_high, loss_scale;
    bf16* dz;          // [M, 256] or nullptr
    float* logp_out;   // may be nullptr
    RowOut out;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], float* scratch) const {
        // scratch (LDS, free after the main loop): [2 quantities][2 column halves][256 rows]
        float* ex_a = scratch;
        float* ex_b = scratch + 512;
        int nk = *n_kept;
        nk = nk < 0 ? 0 : (nk > max_chunks ? max_chunks : nk);
        const int64_t rows_live = (int64_t)nk * A;
        const int lrow_base = tc.wm * 128 + (tc.lane & 31);

        float mx[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) m = fmaxf(m, acc[i][j][e]);
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            mx[i] = m;
            if (tc.lane < 32) ex_a[tc.wn * 256 + lrow_base + i * 32] = m;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) mx[i] = fmaxf(mx[i], ex_a[(tc.wn ^ 1) * 256 + lrow_base + i * 32]);
        __syncthreads();

        float lse[4], ztok[4];
        int tok[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tok[i] = token[tc.row(i)];
            float se = 0.f, zt = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = tc.col(j, q);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float z = acc[i][j][4 * q + t];
                        se += __expf(z - mx[i]);
                        zt += (n + t == tok[i]) ? z : 0.f;
                    }
                }
            se += __shfl_xor(se, 32, 64);
            zt += __shfl_xor(zt, 32, 64);
            lse[i] = se;
            ztok[i] = zt;
            if (tc.lane < 32) {
                ex_a[tc.wn * 256 + lrow_base + i * 32] = se;
                ex_b[tc.wn * 256 + lrow_base + i * 32] = zt;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int other = (tc.wn ^ 1) * 256 + lrow_base + i * 32;
            lse[i] = mx[i] + __logf(lse[i] + ex_a[other]);
            ztok[i] += ex_b[other];
        }

#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
            const bool live = m < rows_live;
            const float lp = ztok[i] - lse[i];
            const LossRow lr = loss_row(lp, logp_old[m], adv_row[m], eps_low, eps_high, loss_scale);
            if (tc.wn == 0 && tc.lane < 32) {
                out.term[m] = live ? lr.term : 0.f;
                out.ratio[m] = lr.ratio;
                out.dlogp[m] = lr.dlogp;
                out.clipped[m] = lr.clipped;
                if (logp_out && live) logp_out[m] = lp;
            }
            if (dz) {
                const float coef = live ? lr.coef : 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = tc.col(j, q);
                        float g[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float pr = __expf(acc[i][j][4 * q + t] - lse[i]);
                            g[t] = coef * (((n + t == tok[i]) ? 1.f : 0.f) - pr);
                        }
                        *reinterpret_cast<bf16x4*>(dz + (int64_t)m * 256 + n) = to_bf16x4(g[0], g[1], g[2], g[3]);
                    }
            }
        }
    }
};

template <class Epilogue>
inline void launch_gemm(const GemmProblem& p, const Epilogue& epi, hipStream_t s) {
    const unsigned grid = (unsigned)(p.M / kTileM) * (unsigned)(p.N / kTileN) * (unsigned)p.splits;
    gemm_bf16_nt<Epilogue><<<grid, kGemmThreads, 0, s>>>(p, epi);
}

}  // namespace pcm
