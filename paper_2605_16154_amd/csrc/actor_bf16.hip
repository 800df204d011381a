// bf16 path of the masked GRPO actor step (Eq. 11): matrix-core GEMMs with fused epilogues.
//
// Forward:  X -> [gate|up] GEMM with silu(u)*v fused -> down GEMM -> logit GEMM with the
//           log-softmax / ratio / clipped surrogate / dz fused.
// Backward: dy = dz Wo^T; da = dy Wd^T with the gated-activation derivative fused (du, dv
//           overwrite the two factors the forward epilogue stored); weight gradients reduce over
//           the row dimension (a small output, dWo, as partial products over slices of the rows,
//           summed afterwards: no atomics); dX = du Wg^T + dv Wu^T as one GEMM over two
//           reduction segments.
// Composed evaluation (an option): the down and the logit projection as the one matrix
//           W_do = Wd Wo [ff, V] formed at the start of the call: z = a W_do; G = a^T dz,
//           dWd = G Wo^T, dWo = Wd^T G, da = dz W_do^T.  y and dy are never formed; the three
//           products through d shrink to products through V.
//
// The forward and input-gradient products take both operands reduction-contiguous; for the forward
// pass the [in, out] weights are first copied transposed (gate and up interleaved in blocks of 64
// columns so that the activation can be fused).  The weight-gradient products reduce over the row
// dimension and read the activations as they are, through the GEMM's LDS transpose reads.
//
// Rows are padded to a multiple of 256; padding rows are zero with zero advantage, so they
// contribute nothing to any output.
//
// Backward over the rows that carry a gradient: a row whose ratio the clip cuts (or whose advantage or weight is
// zero) has an all-zero row of dz, hence of dy, du, dv and dX, and adds nothing to a weight gradient.  After the loss
// a kernel lists the other rows; when at least one row in sixteen drops out, dz, y, a and X are copied row by row
// into dense matrices of the listed rows and every backward product runs over those (the da epilogue reads its
// factors through the list, dX is written through it, its other rows zero-filled).  The decision, the row count and
// the operand addresses stay in device memory: no host synchronisation.  Without an entropy bonus only (with one,
// every row has a gradient), and not in the composed evaluation.
//
// A long batch is worked through in row panels (kPanelRows rows, a multiple of both the tile height
// and the chunk length): gather, forward, loss and backward run panel by panel over the same
// activation buffers, the weight gradients of every panel after the first are added to what the
// earlier ones left, and the per-row loss terms are reduced once at the end.  The workspace is then
// bounded by the panel (about 5 GB at d = 4096, ff = 11008) instead of growing with the batch, and
// a panel's activations are still in the memory-side cache when its backward pass reads them.
#include "gemm_bf16.h"

namespace pcm {
namespace {

constexpr int kPackNone = 0, kPackGate = 1, kPackUp = 2;
constexpr size_t kMaxSplitTiles = 256;   // tiles x parts of a split reduction: one workgroup per CU
constexpr size_t kSumBlocksMax = 2048;   // workgroups of sum_parts_f32 at most

__device__ inline int packed_row(int c, int mode) {
    if (mode == kPackNone) return c;
    return (c / 64) * 128 + (c % 64) + (mode == kPackUp ? 64 : 0);
}

// dst[map(c), r] = src[r, c] for a [R, C] bf16 matrix (R, C multiples of 64); 64 x 64 tiles.
__global__ __launch_bounds__(256) void transpose_bf16(const uint16_t* __restrict__ src, int64_t ld_src,
                                                      uint16_t* __restrict__ dst, int64_t ld_dst, int mode) {
    __shared__ uint16_t tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int t = threadIdx.x, tr = t >> 4, tv = t & 15;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = tr + 16 * q;
        const uint2 v = *reinterpret_cast<const uint2*>(src + (int64_t)(r0 + row) * ld_src + c0 + tv * 4);
        tile[row][tv * 4 + 0] = (uint16_t)(v.x & 0xFFFF);
        tile[row][tv * 4 + 1] = (uint16_t)(v.x >> 16);
        tile[row][tv * 4 + 2] = (uint16_t)(v.y & 0xFFFF);
        tile[row][tv * 4 + 3] = (uint16_t)(v.y >> 16);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = tr + 16 * q;
        uint2 v;
        v.x = (uint32_t)tile[tv * 4 + 0][c] | ((uint32_t)tile[tv * 4 + 1][c] << 16);
        v.y = (uint32_t)tile[tv * 4 + 2][c] | ((uint32_t)tile[tv * 4 + 3][c] << 16);
        *reinterpret_cast<uint2*>(dst + (int64_t)packed_row(c0 + c, mode) * ld_dst + r0 + tv * 4) = v;
    }
}

void transpose(hipStream_t s, const bf16* src, int R, int C, bf16* dst, int64_t ld_dst, int mode, int stage) {
    StageTimer t(stage, s);
    dim3 grid(C / 64, R / 64);
    transpose_bf16<<<grid, 256, 0, s>>>(reinterpret_cast<const uint16_t*>(src), C,
                                        reinterpret_cast<uint16_t*>(dst), ld_dst, mode);
}

__global__ void fill_zero_f64(double* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

// Sum over a workgroup of 256 threads (every thread gets the result).
__device__ inline double block_sum_256(double x) {
    __shared__ double wave_part[4];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = x;
    __syncthreads();
    return wave_part[0] + wave_part[1] + wave_part[2] + wave_part[3];
}

// out[i] = sum over the parts of a split reduction (n is a multiple of 4; parts are n floats apart); kAdd: added
// to what out holds.  With sumsq_parts, on the final panel, every workgroup also writes the sum of the squares of
// the values it left in out to sumsq_parts[workgroup].
template <bool kAdd>
__global__ __launch_bounds__(256) void sum_parts_f32(const float* parts, int n_parts, size_t n, float* out, double* sumsq_parts,
                                                     FinalPanel final_panel) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    double sq = 0.0;
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
        float4 acc = kAdd ? *reinterpret_cast<const float4*>(out + i) : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s = 0; s < n_parts; ++s) {
            const float4 v = *reinterpret_cast<const float4*>(parts + (size_t)s * n + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<float4*>(out + i) = acc;
        sq += (double)acc.x * acc.x + (double)acc.y * acc.y + (double)acc.z * acc.z + (double)acc.w * acc.w;
    }
    if (sumsq_parts != nullptr && final_panel()) {
        sq = block_sum_256(sq);
        if (threadIdx.x == 0) sumsq_parts[blockIdx.x] = sq;
    }
}

// The same sum, rounded once to bf16 (a product that the next GEMM takes as an operand).
__global__ void sum_parts_bf16(const float* parts, int n_parts, size_t n, bf16* out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
        float4 acc = *reinterpret_cast<const float4*>(parts + i);
        for (int s = 1; s < n_parts; ++s) {
            const float4 v = *reinterpret_cast<const float4*>(parts + (size_t)s * n + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        out[i] = __float2bfloat16(acc.x);
        out[i + 1] = __float2bfloat16(acc.y);
        out[i + 2] = __float2bfloat16(acc.z);
        out[i + 3] = __float2bfloat16(acc.w);
    }
}

// The forward products' operand layouts of the four weight matrices, in one buffer.
struct PackedHead {
    bf16 *WguT, *WdT, *WoT;
    size_t bytes;
};
PackedHead carve_packed(void* base, int d, int ff, int V) {
    Carver c(base);
    PackedHead p;
    p.WguT = c.take<bf16>((size_t)2 * ff * d);
    p.WdT = c.take<bf16>((size_t)d * ff);
    p.WoT = c.take<bf16>((size_t)V * d);
    p.bytes = c.used();
    return p;
}

constexpr int64_t kPanelRows = 57344;   // target height of a row panel (224 row tiles)

// Height of the row panels a batch of `sh.rows_max()` rows is worked through in: the whole (padded) batch if it
// is at most a panel and a quarter, or if the head is evaluated in composed form; otherwise the largest common
// multiple of the tile height and the chunk length that does not exceed the target (the caller's, else kPanelRows).
int64_t panel_rows(const ActorShape& sh, bool composed, int target) {
    const int64_t Mp = ceil_div64(sh.rows_max(), kTileM) * kTileM;
    if (composed) return Mp;
    const int64_t want = target > 0 ? target : kPanelRows;
    int64_t x = kTileM, y = sh.A;
    while (y != 0) { const int64_t t = x % y; x = y; y = t; }             // gcd
    const int64_t unit = (int64_t)kTileM / x * sh.A;                        // lcm(256, A)
    const int64_t rp = unit * (want / unit > 0 ? want / unit : 1);
    return Mp <= rp + rp / 4 ? Mp : rp;
}

struct Bf16Workspace {
    bf16 *WguT, *WdT, *WoT;
    bf16 *X, *fu, *fv, *a, *y, *dz, *dz_extra;   // one panel each; fu, fv: SwiGLU derivative factors, then du, dv
    bf16 *a_lo, *y_lo;                           // per-chunk ratio: rounding remainders of a and y
    bf16* dy;
    bf16 *du, *xy, *dzc;   // backward over listed rows: du (before that the listed rows of a), the listed rows of y and
                           // later of X, the listed rows of dz; dv takes the place of a
    int32_t* live_idx;     // [Rp] the listed rows
    LivePlan* plan;        // null: backward over all rows
    double* sumsq[4];      // sums of squares of the final dWg, dWu, dWd, dWo by workgroup (null: not asked for)
    int sumsq_count[4];
    bf16 *Wdo, *G;  // composed evaluation: Wd Wo and a^T dz, both [ff, V]
    float* parts;   // partial products of split reductions
    RowMeta meta;   // whole batch
    RowOut out;     // whole batch
    int64_t Mp;     // padded rows of the batch
    int64_t Rp;     // rows of a panel
    size_t bytes;
};

// Whether the backward products of a call run over the listed rows (see the head of this file).
bool lists_live_rows(const LossOptions& opt, bool bwd, bool composed) {
    return bwd && !composed && !opt.dense_backward && opt.entropy_coef == 0.f;
}

Bf16Workspace carve(void* ws, const ActorShape& sh, bool bwd, bool grads, const LossOptions& opt, bool composed) {
    Carver c(ws);
    Bf16Workspace w{};
    const bool split = opt.chunk_ratio != 0;
    const int panel_target = opt.panel_rows;
    const size_t Mp = (size_t)ceil_div64(sh.rows_max(), kTileM) * kTileM;
    const size_t Rp = (size_t)panel_rows(sh, composed, panel_target);
    const size_t d = sh.d, ff = sh.ff, V = sh.V;
    w.Mp = (int64_t)Mp;
    w.Rp = (int64_t)Rp;
    w.WguT = c.take<bf16>(2 * ff * d);
    w.WdT = c.take<bf16>(d * ff);
    w.WoT = c.take<bf16>(V * d);
    w.X = c.take<bf16>(Rp * d);
    w.a = c.take<bf16>(Rp * ff);
    if (bwd) w.fu = c.take<bf16>(Rp * ff);
    if (bwd) w.fv = c.take<bf16>(Rp * ff);
    w.y = c.take<bf16>(Rp * d);
    if (split) w.a_lo = c.take<bf16>(Rp * ff);
    if (split) w.y_lo = c.take<bf16>(Rp * d);
    w.dz = c.take<bf16>(Rp * V);
    w.meta.token = c.take<uint8_t>(Mp);
    w.meta.logp_old = c.take<float>(Mp);
    w.meta.adv = c.take<float>(Mp);
    w.out.term = c.take<float>(Mp);
    w.out.ratio = c.take<float>(Mp);
    w.out.dlogp = c.take<float>(Mp);
    w.out.clipped = c.take<uint8_t>(Mp);
    w.out.entropy = c.take<float>(Mp);
    w.out.coef = c.take<float>(Mp);
    if (bwd) w.dz_extra = c.take<bf16>(Rp * V);
    if (bwd) w.dy = c.take<bf16>(Rp * d);
    if (lists_live_rows(opt, bwd, composed)) {
        w.du = c.take<bf16>(Rp * ff);
        w.xy = c.take<bf16>(Rp * d);
        w.dzc = c.take<bf16>(Rp * V);
        w.live_idx = c.take<int32_t>(Rp);
        w.plan = c.take<LivePlan>(1);
    }
    if (grads && opt.grad_sumsq_out != nullptr) {
        const size_t tiles[4] = {d / kTileM * (ff / kTileN), d / kTileM * (ff / kTileN), ff / kTileM * (d / kTileN),
                                 d / kTileM * (V / kTileN)};
        for (int q = 0; q < 4; ++q) {
            w.sumsq_count[q] = (int)(4 * tiles[q] > kSumBlocksMax ? 4 * tiles[q] : kSumBlocksMax);
            w.sumsq[q] = c.take<double>((size_t)w.sumsq_count[q]);
        }
    }
    w.Wdo = c.take<bf16>(ff * V);
    if (grads) w.G = c.take<bf16>(ff * V);
    w.parts = c.take<float>(kMaxSplitTiles * (size_t)kTileM * kTileN);
    w.bytes = c.used();
    return w;
}

// Reduction split for an output of `tiles` tiles and `steps` 64-wide reduction steps.  An output
// that already covers the 256 CUs is not split; a small output is split so that tiles * splits
// fills the chip (and never exceeds kMaxSplitTiles, which sizes the buffer of partial products),
// keeping at least 8 steps per workgroup.
int pick_splits(int tiles, int steps) {
    if (tiles >= 256) return 1;
    int s = (int)kMaxSplitTiles / tiles;
    const int max_s = steps / 8 > 0 ? steps / 8 : 1;
    if (s > max_s) s = max_s;
    return s < 1 ? 1 : s;
}

// Which GEMM dimension runs over the kept rows, so that work beyond the device-side count is skipped; the rows
// are those of a panel that starts at batch row `row_offset`.
struct KeptRows {
    const int32_t* kept;
    int kept_max, rows_per_kept;
    int row_offset;
};

// Where a weight-gradient launch leaves the sums of the squares of its final values: the unsplit GEMM four per
// output tile, the kernel that sums a split reduction one per workgroup (parts == nullptr: nowhere).
struct SumsqTarget {
    double* parts;
    FinalPanel final_panel;
};

// C[M, N] = product of p with a long reduction and possibly a small output: fp32 (C32) or rounded to bf16
// (C16), exactly one of the two given.  A small output is computed as several partial products over slices of
// the reduction, summed by a second kernel (no atomics).  The weight gradients are the case
// kLayA = kLayB = kKByRows: A^T B over the kept rows with both operands stored [rows][features].
// accumulate (fp32 output only): the product is added to C.
template <int kLayA, int kLayB>
void launch_reduction_gemm(GemmProblem p, float* C32, bf16* C16, float* parts, bool accumulate, const SumsqTarget& sq, int stage,
                           hipStream_t s) {
    p.splits = pick_splits((p.M / kTileM) * (p.N / kTileN), p.K1 / kTileK);
    StageTimer t(stage, s);
    if (p.splits == 1) {
        p.skip_if_empty = accumulate ? 1 : 0;
        if (C32) launch_gemm<kLayA, kLayB>(p, EpiStoreF32{C32, p.N, 0, accumulate ? 1 : 0, sq.parts, sq.final_panel}, s);
        else launch_gemm<kLayA, kLayB>(p, EpiStoreBf16{C16, p.N, p.M}, s);
        return;
    }
    const size_t n = (size_t)p.M * p.N;
    launch_gemm<kLayA, kLayB>(p, EpiStoreF32{parts, p.N, (int64_t)n, 0, nullptr, FinalPanel{}}, s);
    size_t blocks = (n / 4 + 255) / 256;
    if (blocks > kSumBlocksMax) blocks = kSumBlocksMax;
    if (C32 && accumulate) sum_parts_f32<true><<<(unsigned)blocks, 256, 0, s>>>(parts, p.splits, n, C32, sq.parts, sq.final_panel);
    else if (C32) sum_parts_f32<false><<<(unsigned)blocks, 256, 0, s>>>(parts, p.splits, n, C32, sq.parts, sq.final_panel);
    else sum_parts_bf16<<<(unsigned)blocks, 256, 0, s>>>(parts, p.splits, n, C16);
}
void launch_weight_grad(const GemmProblem& p, float* C, float* parts, bool accumulate, const SumsqTarget& sq, int stage,
                        hipStream_t s) {
    launch_reduction_gemm<kKByRows, kKByRows>(p, C, nullptr, parts, accumulate, sq, stage, s);
}

GemmProblem problem(const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int M, int N, int K,
                    const KeptRows& kr, int rows_role) {
    GemmProblem p{};
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb;
    p.A2 = A; p.B2 = B;
    p.M = M; p.N = N; p.K1 = K; p.K2 = 0; p.splits = 1;
    p.kept = kr.kept; p.kept_max = kr.kept_max; p.rows_per_kept = kr.rows_per_kept; p.rows_role = rows_role;
    p.row_offset = kr.row_offset; p.skip_if_empty = 0;
    return p;
}

}  // namespace

size_t packed_head_bytes(int d, int ff, int V) { return carve_packed(nullptr, d, ff, V).bytes; }

int pack_head_weights(const void* Wg, const void* Wu, const void* Wd, const void* Wo, int d, int ff, int V, void* packed,
                      hipStream_t s) {
    const PackedHead p = carve_packed(packed, d, ff, V);
    transpose(s, static_cast<const bf16*>(Wg), d, ff, p.WguT, d, kPackGate, ST_WEIGHT_LAYOUT);
    transpose(s, static_cast<const bf16*>(Wu), d, ff, p.WguT, d, kPackUp, ST_WEIGHT_LAYOUT);
    transpose(s, static_cast<const bf16*>(Wd), ff, d, p.WdT, ff, kPackNone, ST_WEIGHT_LAYOUT);
    transpose(s, static_cast<const bf16*>(Wo), d, V, p.WoT, d, kPackNone, ST_WEIGHT_LAYOUT);
    return launch_status();
}

size_t actor_bf16_workspace_bytes(const ActorShape& sh, bool want_grads, const LossOptions& opt, bool composed) {
    return carve(nullptr, sh, want_grads, want_grads, opt, composed).bytes;
}

int actor_bf16_run(const ActorShape& sh, const ActorIO& io, void* ws, hipStream_t s) {
    const bool grads = io.want_grads();
    const bool bwd = grads || io.dX != nullptr;
    // With one ratio per chunk the log-probabilities of a chunk's A rows add up in the exponent, and so do their
    // errors: the forward pass then carries a and y as pairs of bf16 values (value and rounding remainder) through
    // the down and the logit product, which brings the error of a log-probability from about 2e-3 down to 1e-5.
    const bool split = io.opt.chunk_ratio != 0;
    Bf16Workspace w = carve(ws, sh, bwd, grads, io.opt, io.composed);
    const int d = sh.d, ff = sh.ff, V = sh.V;
    const bf16* Wg = static_cast<const bf16*>(io.Wg);
    const bf16* Wu = static_cast<const bf16*>(io.Wu);
    const bf16* Wd = static_cast<const bf16*>(io.Wd);
    const bf16* Wo = static_cast<const bf16*>(io.Wo);

    const KeptRows all_rows{nullptr, 0, 0, 0};
    if (io.opt.packed_weights != nullptr) {               // layouts kept by the caller: nothing to re-lay-out
        const PackedHead ph = carve_packed(const_cast<void*>(io.opt.packed_weights), d, ff, V);
        w.WguT = ph.WguT; w.WdT = ph.WdT; w.WoT = ph.WoT;
    } else {
        transpose(s, Wg, d, ff, w.WguT, d, kPackGate, ST_WEIGHT_LAYOUT);   // [d, ff] -> packed rows of [2 ff, d]
        transpose(s, Wu, d, ff, w.WguT, d, kPackUp, ST_WEIGHT_LAYOUT);
        if (io.composed) {
            // W_do = Wd Wo [ff, V], from the weights as given (Wd [rows][K], Wo [K][rows])
            launch_reduction_gemm<kRowsByK, kKByRows>(problem(Wd, d, Wo, V, ff, V, d, all_rows, kRowsUnused), nullptr, w.Wdo,
                                                      w.parts, false, SumsqTarget{}, ST_WEIGHT_LAYOUT, s);
        } else {
            transpose(s, Wd, ff, d, w.WdT, ff, kPackNone, ST_WEIGHT_LAYOUT);   // [ff, d] -> [d, ff]
            transpose(s, Wo, d, V, w.WoT, d, kPackNone, ST_WEIGHT_LAYOUT);     // [d, V]  -> [V, d]
        }
    }

    const bool want_sumsq = grads && io.opt.grad_sumsq_out != nullptr && ws != nullptr && w.sumsq[0] != nullptr;
    if (want_sumsq)   // slots no launch of this call writes must read as zero (a fill kernel: safe under graph capture)
        for (int q = 0; q < 4; ++q) fill_zero_f64<<<(w.sumsq_count[q] + 255) / 256, 256, 0, s>>>(w.sumsq[q], w.sumsq_count[q]);

    int rc = PCM_OK;
    for (int64_t row0 = 0; row0 < w.Mp; row0 += w.Rp) {
        // this panel: batch rows [row0, row0 + Mp); all row-indexed arrays below are its parts
        const int Mp = (int)(w.Mp - row0 < w.Rp ? w.Mp - row0 : w.Rp);
        const bool first = row0 == 0;
        const KeptRows kr{io.n_kept, sh.max_chunks, sh.A, (int)row0};
        SumsqTarget sq[4] = {};    // dWg, dWu, dWd, dWo
        if (want_sumsq) {
            const FinalPanel fp{io.n_kept, sh.max_chunks, sh.A, row0, row0 + w.Rp >= w.Mp ? INT64_MAX : row0 + w.Rp};
            for (int q = 0; q < 4; ++q) sq[q] = SumsqTarget{w.sumsq[q], fp};
        }
        const RowMeta meta{w.meta.token + row0, w.meta.logp_old + row0, w.meta.adv + row0};
        const RowOut out{w.out.term + row0, w.out.ratio + row0, w.out.dlogp + row0, w.out.clipped + row0,
                         w.out.entropy + row0, w.out.coef + row0};
        rc = launch_gather(sh, io, 2, w.X, row0, Mp, meta, s);
        if (rc != PCM_OK) return rc;
        {
            StageTimer t(ST_GEMM_GATE_UP, s);
            const GemmProblem p = problem(w.X, d, w.WguT, d, Mp, 2 * ff, d, kr, kRowsAreM);
            if (split && bwd) launch_gemm(p, EpiSwigluForward<true, true>{w.fu, w.fv, w.a, w.a_lo, ff}, s);
            else if (split) launch_gemm(p, EpiSwigluForward<false, true>{nullptr, nullptr, w.a, w.a_lo, ff}, s);
            else if (bwd) launch_gemm(p, EpiSwigluForward<true>{w.fu, w.fv, w.a, nullptr, ff}, s);
            else launch_gemm(p, EpiSwigluForward<false>{nullptr, nullptr, w.a, nullptr, ff}, s);
        }
        if (!io.composed) {
            StageTimer t(ST_GEMM_DOWN, s);
            GemmProblem p = problem(w.a, ff, w.WdT, ff, Mp, d, ff, kr, kRowsAreM);
            if (split) {                                       // y = [a | a_lo] [Wd; Wd], kept as y + y_lo
                p.A2 = w.a_lo; p.B2 = w.WdT; p.K2 = ff;
                launch_gemm(p, EpiStoreBf16Split{w.y, w.y_lo, d, Mp}, s);
            } else {
                launch_gemm(p, EpiStoreBf16{w.y, d, Mp}, s);
            }
        }
        {
            StageTimer t(ST_GEMM_LOGITS_LOSS, s);
            EpiLogitsLoss epi{meta.token, meta.logp_old, meta.adv, io.n_kept, sh.max_chunks, sh.A, (int)row0,
                              io.opt, bwd ? w.dz : nullptr, w.dz_extra, io.logp_out ? io.logp_out + row0 : nullptr, out};
            if (io.composed) {   // z = a W_do, W_do read as [K][rows]
                launch_gemm<kRowsByK, kKByRows>(problem(w.a, ff, w.Wdo, V, Mp, V, ff, kr, kRowsAreM), epi, s);
            } else {
                GemmProblem p = problem(w.y, d, w.WoT, d, Mp, V, d, kr, kRowsAreM);
                if (split) { p.A2 = w.y_lo; p.B2 = w.WoT; p.K2 = d; }   // z = [y | y_lo] [Wo; Wo]
                launch_gemm(p, epi, s);
            }
        }
        if (io.opt.chunk_ratio) {
            rc = launch_chunk_ratio(sh, io, meta, out, row0, Mp, s);
            if (rc != PCM_OK) return rc;
            if (bwd) {
                rc = launch_scale_rows(sh, io, w.dz, io.opt.entropy_coef != 0.f ? w.dz_extra : nullptr, out.coef, row0, Mp,
                                       2, s);
                if (rc != PCM_OK) return rc;
            }
        }
        if (!bwd) continue;

        if (w.plan != nullptr) {
            // backward over the rows with a gradient; row counts and row-indexed operands come from the plan
            const bf16* const* const src = reinterpret_cast<const bf16* const*>(w.plan->src);
            const KeptRows lr{&w.plan->n_rows, Mp, 1, 0};
            bf16* const dv = w.a;                       // free once the listed rows of a are copied
            {
                StageTimer t(ST_LIVE_ROWS, s);
                const LiveSources whole{{w.dz, w.y, w.a, w.X}}, listed{{w.dzc, w.xy, w.du, w.xy}};
                rc = launch_live_row_list(sh, io, out.clipped, meta.adv, row0, Mp, whole, listed, w.live_idx, w.plan, s);
                if (rc != PCM_OK) return rc;
                launch_gather_listed(w.dz, w.live_idx, w.plan, Mp, (int64_t)V * 2, w.dzc, s);
                if (grads) launch_gather_listed(w.y, w.live_idx, w.plan, Mp, (int64_t)d * 2, w.xy, s);
                if (grads) launch_gather_listed(w.a, w.live_idx, w.plan, Mp, (int64_t)ff * 2, w.du, s);
            }
            {
                StageTimer t(ST_GEMM_DY, s);
                GemmProblem p = problem(w.dz, V, Wo, V, Mp, d, V, lr, kRowsAreM);                                // dy = dz Wo^T
                p.A_sel = src + LiveSources::kDz;
                launch_gemm(p, EpiStoreBf16{w.dy, d, Mp}, s);
            }
            if (grads) {
                GemmProblem p = problem(w.y, d, w.dz, V, d, V, Mp, lr, kRowsAreK);                               // dWo (+)= y^T dz
                p.A_sel = src + LiveSources::kY;
                p.B_sel = src + LiveSources::kDz;
                launch_weight_grad(p, io.dWo, w.parts, !first, sq[3], ST_GEMM_DWO, s);
                p = problem(w.a, ff, w.dy, d, ff, d, Mp, lr, kRowsAreK);                                         // dWd (+)= a^T dy
                p.A_sel = src + LiveSources::kA;
                launch_weight_grad(p, io.dWd, w.parts, !first, sq[2], ST_GEMM_DWD, s);
            }
            {
                StageTimer t(ST_GEMM_DA, s);                                                                     // du, dv from da = dy Wd^T
                launch_gemm(problem(w.dy, d, Wd, d, Mp, ff, d, lr, kRowsAreM),
                            EpiSwigluBackward<true>{w.fu, w.fv, ff, w.live_idx, w.du, dv}, s);
            }
            if (grads) {
                {
                    StageTimer t(ST_LIVE_ROWS, s);
                    launch_gather_listed(w.X, w.live_idx, w.plan, Mp, (int64_t)d * 2, w.xy, s);
                }
                GemmProblem p = problem(w.X, d, w.du, ff, d, ff, Mp, lr, kRowsAreK);                             // dWg (+)= X^T du
                p.A_sel = src + LiveSources::kX;
                launch_weight_grad(p, io.dWg, w.parts, !first, sq[0], ST_GEMM_DWG_DWU, s);
                p.B = dv;                                                                                        // dWu (+)= X^T dv
                p.B2 = dv;
                launch_weight_grad(p, io.dWu, w.parts, !first, sq[1], ST_GEMM_DWG_DWU, s);
            }
            if (io.dX) {
                const int64_t rows_left = sh.rows_max() - row0;
                bf16* const dX = static_cast<bf16*>(io.dX) + row0 * d;
                {
                    StageTimer t(ST_LIVE_ROWS, s);
                    rc = launch_zero_unlisted(sh, io, out.clipped, meta.adv, row0, Mp, rows_left < Mp ? rows_left : Mp, (int64_t)d * 2, dX,
                                              s);
                    if (rc != PCM_OK) return rc;
                }
                StageTimer t(ST_GEMM_DX, s);
                GemmProblem p = problem(w.du, ff, Wg, ff, Mp, d, ff, lr, kRowsAreM);                             // dX = du Wg^T + dv Wu^T
                p.A2 = dv; p.B2 = Wu; p.K2 = ff;
                launch_gemm(p, EpiScatterBf16{dX, d, w.live_idx}, s);
            }
            continue;
        }
        if (io.composed) {      // one panel: nothing to add to
            if (grads) {
                // G = a^T dz [ff, V] over the kept rows, rounded to bf16 as the operand of the two products below
                launch_reduction_gemm<kKByRows, kKByRows>(problem(w.a, ff, w.dz, V, ff, V, Mp, kr, kRowsAreK), nullptr, w.G,
                                                          w.parts, false, SumsqTarget{}, ST_GEMM_DWD, s);
                {
                    StageTimer t(ST_GEMM_DWD, s);                                                                 // dWd = G Wo^T
                    launch_gemm<kRowsByK, kRowsByK>(problem(w.G, V, Wo, V, ff, d, V, all_rows, kRowsUnused),
                                                    EpiStoreF32{io.dWd, d, 0, 0, nullptr, FinalPanel{}}, s);
                }
                launch_weight_grad(problem(Wd, d, w.G, V, d, V, ff, all_rows, kRowsUnused), io.dWo, w.parts, false,
                                   SumsqTarget{}, ST_GEMM_DWO, s);                                                               // dWo = Wd^T G
            }
            StageTimer t(ST_GEMM_DA, s);                                                                          // da = dz W_do^T
            launch_gemm(problem(w.dz, V, w.Wdo, V, Mp, ff, V, kr, kRowsAreM), EpiSwigluBackward<false>{w.fu, w.fv, ff, nullptr, nullptr, nullptr}, s);
        } else {
            {
                StageTimer t(ST_GEMM_DY, s);
                launch_gemm(problem(w.dz, V, Wo, V, Mp, d, V, kr, kRowsAreM), EpiStoreBf16{w.dy, d, Mp}, s);          // dy = dz Wo^T
            }
            if (grads) {
                launch_weight_grad(problem(w.y, d, w.dz, V, d, V, Mp, kr, kRowsAreK), io.dWo, w.parts, !first, sq[3],
                                   ST_GEMM_DWO, s);                                                                            // dWo (+)= y^T dz
                launch_weight_grad(problem(w.a, ff, w.dy, d, ff, d, Mp, kr, kRowsAreK), io.dWd, w.parts, !first, sq[2],
                                   ST_GEMM_DWD, s);                                                                            // dWd (+)= a^T dy
            }
            StageTimer t(ST_GEMM_DA, s);
            launch_gemm(problem(w.dy, d, Wd, d, Mp, ff, d, kr, kRowsAreM), EpiSwigluBackward<false>{w.fu, w.fv, ff, nullptr, nullptr, nullptr}, s);   // fu <- du, fv <- dv
        }
        if (grads) {
            launch_weight_grad(problem(w.X, d, w.fu, ff, d, ff, Mp, kr, kRowsAreK), io.dWg, w.parts, !first, sq[0],
                               ST_GEMM_DWG_DWU, s);                                                                                // dWg (+)= X^T du
            launch_weight_grad(problem(w.X, d, w.fv, ff, d, ff, Mp, kr, kRowsAreK), io.dWu, w.parts, !first, sq[1],
                               ST_GEMM_DWG_DWU, s);                                                                                // dWu (+)= X^T dv
        }
        if (io.dX) {
            StageTimer t(ST_GEMM_DX, s);
            GemmProblem p = problem(w.fu, ff, Wg, ff, Mp, d, ff, kr, kRowsAreM);                                 // dX = du Wg^T + dv Wu^T
            p.A2 = w.fv; p.B2 = Wu; p.K2 = ff;
            const int64_t rows_left = sh.rows_max() - row0;
            launch_gemm(p, EpiStoreBf16{static_cast<bf16*>(io.dX) + row0 * d, d, (int)(rows_left < Mp ? rows_left : Mp)}, s);
        }
    }
    SumsqLists lists{};
    if (want_sumsq)
        for (int q = 0; q < 4; ++q) { lists.parts[q] = w.sumsq[q]; lists.count[q] = w.sumsq_count[q]; }
    rc = launch_loss_reduce(sh, io, w.out, lists, s);
    if (rc != PCM_OK) return rc;
    return launch_status();
}

}  // namespace pcm
