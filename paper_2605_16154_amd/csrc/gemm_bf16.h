// bf16 matrix-core GEMM for gfx950 with fused epilogues (internal header).
//
// C[m, n] = sum_k A(m, k) * B(n, k).  Each operand may be stored either with the reduction index
// contiguous ([rows][K], the layout the MFMA operand registers want: a lane feeds 8 consecutive k
// of one row, read with ds_read_b128) or with the reduction index as the slow dimension
// ([K][rows], e.g. activations in the weight-gradient products); the latter is brought into
// operand layout by gfx950's LDS transpose reads (ds_read_b64_tr_b16), so no operand is ever
// copied transposed in memory.
//
// Tiling: 256 x 256 x 64 per workgroup of 4 wavefronts (2 x 2), each wavefront owning 128 x 128 =
// 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 with fp32 accumulators (256 accumulator registers per
// lane, one wavefront per SIMD).  Operand tiles (32 KB each) live in a ring of five LDS slots
// filled by direct global-to-LDS loads (no staging registers): two slots are being multiplied,
// up to three are in flight, so the load path never drains at the per-step barrier.  Rows are
// 128 B and the eight 16-byte pieces of a row are XOR-swizzled with the row index so that the
// 16-byte fragment reads spread over all banks.
//
// The MFMA is issued with the B fragment as the first operand, so the accumulator tile is the
// transpose of the usual one: a lane holds, for one output row m, runs of 4 consecutive n.
// Epilogues therefore see 4-wide row-contiguous vectors (8-byte writes into the staging area,
// from which whole rows leave as 16-byte-per-lane stores).
#pragma once

#include "actor.h"

namespace pcm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// How an operand of C[m, n] = sum_k A(m, k) B(n, k) is stored.
enum OperandLayout : int {
    kRowsByK = 0,   // [rows][K]: element (row, k) at ptr[row * ld + k]
    kKByRows = 1    // [K][rows]: element (row, k) at ptr[k * ld + row]
};

constexpr int kTileM = 256, kTileN = 256, kTileK = 64;
constexpr int kGemmThreads = 256;
constexpr int kNumXcd = 8;
constexpr int kRingSlots = 5;    // operand tiles resident or in flight in LDS
// Epilogues pass their results through LDS so that global stores are whole 128-byte lines: each
// wavefront owns a private staging area (no workgroup barrier needed; LDS operations of one
// wavefront execute in order).
constexpr int kWaveStageBytes = 33792;                       // 128 rows x (256 + 8) bytes
constexpr int kSmemBytes = kRingSlots * kTileM * kTileK * 2;   // 160 KB: the whole LDS of a CU
static_assert(4 * kWaveStageBytes <= kSmemBytes, "epilogue staging must fit in the operand ring");

struct GemmProblem {
    const bf16* A;    // M x K1 operand, leading dimension lda (layout given by the kernel's template arguments)
    const bf16* B;    // N x K1 operand, leading dimension ldb
    const bf16* A2;   // optional second reduction segment (same M, N, layouts and leading dimensions), K2 columns;
    const bf16* B2;   // when K2 == 0 both must still point at valid operands (A, B)
    int64_t lda, ldb;
    int M, N, K1, K2;  // M, N multiples of 256; K1, K2 multiples of 64
    int splits;        // reduction split (grid multiplies by it); epilogue must combine partials
    // Device-side row count: when `kept` is set, only the first min(*kept, kept_max) * rows_per_kept
    // rows of the row dimension carry data.  rows_role says which GEMM dimension that is:
    // kRowsAreM: row tiles entirely beyond the count exit at once; kRowsAreK: the reduction stops at
    // the count rounded up to a whole step (rows up to there are valid, zero-padded).
    // With row_offset the operand rows are a panel of a longer batch: the panel's live rows are the batch's live
    // rows beyond row_offset.  skip_if_empty: a workgroup whose reduction range is empty leaves without running the
    // epilogue (for epilogues that add to what is already there).
    const int32_t* kept;
    int kept_max, rows_per_kept, rows_role;
    int row_offset, skip_if_empty;
    // Operands chosen on the device: when set, the first-segment operand is read from *A_sel (*B_sel) instead of A
    // (B); an earlier kernel of the same stream decides which buffer that is.  Single reduction segment only.
    const bf16* const* A_sel;
    const bf16* const* B_sel;
};
enum RowsRole : int { kRowsUnused = 0, kRowsAreM = 1, kRowsAreK = 2 };

// Accumulator coordinates.  For tile (i, j) of the wavefront and register e = 4 * q + t:
//   row  m = m0 + wm * 128 + i * 32 + (lane & 31)
//   col  n = n0 + wn * 128 + j * 32 + 8 * q + 4 * (lane >> 5) + t
struct TileCoord {
    int m0, n0, wm, wn, lane;
    int split;   // which part of a split reduction this workgroup computed
    __device__ int row(int i) const { return m0 + wm * 128 + i * 32 + (lane & 31); }
    __device__ int col(int j, int q) const { return n0 + wn * 128 + j * 32 + 8 * q + 4 * (lane >> 5); }
};

__device__ inline bf16x4 to_bf16x4(float a, float b, float c, float d) {
    bf16x4 r;
    r[0] = (__bf16)a; r[1] = (__bf16)b; r[2] = (__bf16)c; r[3] = (__bf16)d;
    return r;
}

// LDS has 64 four-byte banks (256 B per cycle), so a 16-byte-per-lane read is served 16 lanes at a
// time and a 128-byte tile row covers half the banks.  [rows][K] tiles: 16 consecutive rows must
// fall on 16 different 16-byte columns of the 256-byte window, hence the XOR with row bits 1..3
// (bit 0 already selects the half window).
__device__ inline int swizzle_piece(int row, int piece) { return piece ^ ((row >> 1) & 7); }
// [K][rows] tiles (512-byte k-rows, read by transpose reads of four k-rows x 32 bytes per 16 lanes,
// 32 lanes per cycle): within a 16-lane group the four k-rows are spread by XOR with k & 3; the two
// groups served together read the same k-rows at adjacent 32-byte units, so bits 0 and 2 of the
// unit index are exchanged to put them in different half windows.  Self-inverse for fixed k.
__device__ inline int swizzle_unit(int unit, int k_low2) {
    const int swapped = ((unit & 1) << 2) | (unit & 2) | ((unit >> 2) & 1) | (unit & 8);
    return swapped ^ k_low2;
}
__device__ inline int unswizzle_unit(int phys, int k_low2) {
    const int t = phys ^ k_low2;
    return ((t & 1) << 2) | (t & 2) | ((t >> 2) & 1) | (t & 8);
}

// Workgroup id -> (tile_m, tile_n), or false if the workgroup has no tile.  Consecutive hardware
// workgroup ids go to different XCDs (id mod 8), each with its own L2.  The live tiles are numbered
// in column-major bands of 4 row-tiles, so that 32 consecutive numbers are a block of 4 x 8 tiles
// (12 operand panels between them); such blocks are dealt to the XCDs in turn.  The 32 workgroups
// that run together on one XCD then share their panels in that XCD's L2, and the eight XCDs work
// side by side on the same band at the same time, so that a panel one of them has brought in from
// HBM is found in the memory-side cache by the others.  (Giving each XCD a contiguous range of tiles
// instead costs 3 % on the gate/up shape: the XCDs then stream eight different bands through the
// memory-side cache at once.)  Of the n_wg workgroups launched only tiles_m * tiles_n have a tile
// (the row dimension may be cut short by a device-side count); only those are numbered, so a short
// batch still spreads over all XCDs.
__device__ inline bool tile_of_workgroup(int wg, int n_wg, int tiles_m, int tiles_n, int& tm, int& tn) {
    (void)n_wg;
    constexpr int kBlock = 32;                      // tiles per XCD block = workgroups resident on one XCD
    const int n_live = tiles_m * tiles_n;
    const int xcd = wg % kNumXcd, idx = wg / kNumXcd;
    const int full = n_live / (kBlock * kNumXcd);   // rounds in which every XCD gets a whole block
    int logical;
    if (idx < full * kBlock) logical = ((idx / kBlock) * kNumXcd + xcd) * kBlock + idx % kBlock;
    else logical = full * kBlock * kNumXcd + (idx - full * kBlock) * kNumXcd + xcd;   // the rest, tile by tile
    if (logical >= n_live) return false;
    constexpr int kBand = 4;
    const int band_size = kBand * tiles_n;
    const int band = logical / band_size;
    const int first = band * kBand;
    const int rows = min(tiles_m - first, kBand);
    const int in_band = logical % band_size;
    tm = first + in_band % rows;
    tn = in_band / rows;
    return true;
}

#define PCM_AS_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PCM_AS_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

// One wave-wide 16-byte-per-lane load from global memory straight into LDS: lane l's 16 bytes land
// at lds_addr + 16 l.  Written as inline assembly so that the compiler does not serialise the
// fragment reads of one stage behind loads into the other; completion is awaited explicitly
// (wait_direct_loads) before the barrier that publishes the stage.
__device__ inline void direct_load_16B(const char* base, uint32_t lane_offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_offset), "s"(base)
                 : "memory");
}
// Direct loads retire in issue order, so waiting until at most `newest` remain outstanding
// guarantees that all older ones have landed.
template <int kNewest>
__device__ inline void wait_direct_loads() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kNewest) : "memory");
}

// 8 bf16 of one operand row at 8 consecutive k, from a [K][rows] tile: two transpose reads of 4 k
// each.  Within a group of 16 lanes the instruction hands lane j the j-th 16-bit element of each of
// the four 32-byte runs addressed by lanes 4 q .. 4 q + 3 (q = 0..3); the callers point run q at
// k-row q, so lane j receives k = 0..3 of row j.
__device__ inline bf16x8 read_transposed_fragment(const char* lds_ptr) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_ptr));
    const s16x4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_ptr + 4 * 512));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// An epilogue may ask to run although the workgroup's reduction range is empty and skip_if_empty is set (it then
// sees a zero accumulator): it says so through a member runs_when_empty().
template <class E>
__device__ inline auto runs_when_empty(const E& e, int) -> decltype(e.runs_when_empty()) { return e.runs_when_empty(); }
template <class E>
__device__ inline bool runs_when_empty(const E&, long) { return false; }

template <class Epilogue, int kLayA, int kLayB>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16(GemmProblem p, Epilogue epi) {
    constexpr int kTileElems = kTileM * kTileK;                  // one operand tile
    constexpr uint32_t kTileBytes = kTileElems * 2;
    constexpr int kLoadsPerTile = 8;                             // wave-wide loads per wavefront per tile
    __shared__ __attribute__((aligned(1024))) __bf16 smem[kSmemBytes / 2];   // [slot][row][64]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_m = p.M / kTileM, tiles_n = p.N / kTileN;
    const int n_tiles = tiles_m * tiles_n;
    const int split = blockIdx.x / n_tiles;
    int k1 = p.K1, live_m = tiles_m;
    if (p.kept != nullptr) {
        int nk = *p.kept;
        nk = nk < 0 ? 0 : (nk > p.kept_max ? p.kept_max : nk);
        const int rows = max(0, nk * p.rows_per_kept - p.row_offset);
        if (p.rows_role == kRowsAreM) live_m = min(tiles_m, (rows + kTileM - 1) / kTileM);
        if (p.rows_role == kRowsAreK) k1 = min(k1, (rows + kTileK - 1) / kTileK * kTileK);
    }
    int tm, tn;
    if (!tile_of_workgroup(blockIdx.x % n_tiles, n_tiles, live_m, tiles_n, tm, tn)) return;   // before any barrier
    const int m0 = tm * kTileM, n0 = tn * kTileN;
    // reduction range of this workgroup, in 64-wide steps over the concatenation of both segments
    const int steps1 = k1 / kTileK, steps_all = steps1 + p.K2 / kTileK;
    const int per_split = (steps_all + p.splits - 1) / p.splits;
    const int step_begin = split * per_split;
    const int step_end = min(steps_all, step_begin + per_split);

    // Global -> LDS: one wave-wide load fills 1 KB of LDS, lane l landing in 16-byte slot l; the
    // swizzle is therefore applied on the global side (the lane that lands in a slot fetches the
    // piece that belongs there).  Addresses are a wave-uniform base (tile origin + k offset) plus
    // a 32-bit per-lane byte offset.
    //   [rows][K] operand: the tile is [256 rows][128 B]; wave w fills rows [64 w, 64 w + 64), 8 rows
    //     per load; piece p of row r sits in slot swizzle_piece(r, p).
    //   [K][rows] operand: the tile is [64 k][512 B]; wave w fills k-rows [16 w, 16 w + 16), 2 per
    //     load; the 32-byte unit u of k-row k sits in unit swizzle_unit(u, k & 3).
    const uint32_t lds_base = (uint32_t)(uintptr_t)PCM_AS_LDS(smem);
    struct LoadCtx {
        const char* base;        // wave-uniform
        uint32_t off[2];         // per-lane byte offset of an even / odd load before the per-load stride
        uint32_t stride;         // bytes between consecutive loads
        uint32_t dst;            // LDS byte address of this wave's part of the slot
    };
    // operand 0 = A rows m0.., operand 1 = B rows n0..  Per-lane offsets do not depend on the step; the
    // tile origin is a wave-uniform pointer that walks along k.
    uint32_t lane_off[2][2], load_stride[2];
    const char* seg_origin[2][2];          // [operand][segment]: this tile's bytes at k = 0 of the segment
    int64_t k_step_bytes[2];               // distance between consecutive steps
#pragma unroll
    for (int operand = 0; operand < 2; ++operand) {
        const uint32_t ld = (uint32_t)(operand == 0 ? p.lda : p.ldb);
        const int row0 = operand == 0 ? m0 : n0;
        const int layout = operand == 0 ? kLayA : kLayB;
        const bf16* const* sel = operand == 0 ? p.A_sel : p.B_sel;
        const bf16* s1 = sel != nullptr ? *sel : (operand == 0 ? p.A : p.B);
        const bf16* s2 = sel != nullptr ? s1 : (operand == 0 ? p.A2 : p.B2);
        if (layout == kRowsByK) {
            const uint32_t row = (uint32_t)wave * 64u + (uint32_t)(lane >> 3);      // + 8 r for load r
#pragma unroll
            for (uint32_t odd = 0; odd < 2; ++odd) {                                 // the swizzle may use row bit 3
                const uint32_t piece = (uint32_t)swizzle_piece((lane >> 3) + 8 * odd, lane & 7);
                lane_off[operand][odd] = (row * ld + piece * 8u) * 2u;
            }
            load_stride[operand] = 16u * ld;
            seg_origin[operand][0] = reinterpret_cast<const char*>(s1 + (int64_t)row0 * ld);
            seg_origin[operand][1] = reinterpret_cast<const char*>(s2 + (int64_t)row0 * ld);
            k_step_bytes[operand] = kTileK * 2;
        } else {
            const uint32_t krow = (uint32_t)wave * 16u + (uint32_t)(lane >> 5);      // + 2 r for load r
#pragma unroll
            for (uint32_t odd = 0; odd < 2; ++odd) {
                const uint32_t k_low = 2u * odd + (uint32_t)(lane >> 5);             // (k-row of the load) & 3
                const uint32_t piece = 2u * (uint32_t)unswizzle_unit((lane & 31) >> 1, (int)k_low) + (uint32_t)(lane & 1);
                lane_off[operand][odd] = (krow * ld + piece * 8u) * 2u;
            }
            load_stride[operand] = 4u * ld;
            seg_origin[operand][0] = reinterpret_cast<const char*>(s1 + row0);
            seg_origin[operand][1] = reinterpret_cast<const char*>(s2 + row0);
            k_step_bytes[operand] = (int64_t)kTileK * ld * 2;
        }
    }
    auto tile_origin = [&](int operand, int step) {
        const bool seg1 = step < steps1;
        return seg_origin[operand][seg1 ? 0 : 1] + (int64_t)(seg1 ? step : step - steps1) * k_step_bytes[operand];
    };
    // `slot` is the byte offset of a ring slot
    auto load_ctx_at = [&](int operand, uint32_t slot, const char* origin) {
        LoadCtx c;
        c.base = origin;
        c.off[0] = lane_off[operand][0];
        c.off[1] = lane_off[operand][1];
        c.stride = load_stride[operand];
        c.dst = lds_base + slot + (uint32_t)wave * 8192u;
        return c;
    };
    auto load_ctx = [&](int operand, uint32_t slot, int step) { return load_ctx_at(operand, slot, tile_origin(operand, step)); };
    auto issue_loads = [&](const LoadCtx& c, uint32_t r0, uint32_t n) {
#pragma unroll
        for (uint32_t r = r0; r < r0 + n; ++r) direct_load_16B(c.base, c.off[r & 1u] + r * c.stride, c.dst + r * 1024u);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Fragment registers are double-buffered: while the 16 MFMAs of one 16-wide k-slice run, the
    // 8 fragment reads of the next slice are in flight.  Fragment pair i = rows 32 i .. 32 i + 31 of
    // the wavefront's A and B sub-tiles.
    bf16x8 fa[2][4], fb[2][4];
    // byte offset inside a tile of this lane's fragment for row block i, slice ks
    auto frag_offset = [&](int layout, int sub_row0, int ks, int i) -> uint32_t {
        if (layout == kRowsByK) {
            const int row = sub_row0 + i * 32 + (lane & 31);
            const int piece = ks * 2 + (lane >> 5);
            return (uint32_t)(row * (kTileK * 2) + swizzle_piece(row, piece) * 16);
        }
        const int g = lane >> 4, j = lane & 15;                    // 16-lane group, lane in group
        const int col0 = sub_row0 + i * 32 + (g & 1) * 16;         // this group's 16 rows of the operand
        const int k = ks * 16 + (g >> 1) * 8 + (j >> 2);           // k-row this lane's run starts in
        return (uint32_t)(k * 512 + (swizzle_unit(col0 >> 4, j >> 2) << 5) + ((j & 3) << 3));
    };
    auto read_frag_a = [&](int set, uint32_t slot_a, int ks, int i) {
        const char* sa = reinterpret_cast<const char*>(smem) + slot_a + frag_offset(kLayA, wm * 128, ks, i);
        if (kLayA == kRowsByK) fa[set][i] = *reinterpret_cast<const bf16x8*>(sa);
        else fa[set][i] = read_transposed_fragment(sa);
    };
    auto read_frag_b = [&](int set, uint32_t slot_b, int ks, int j) {
        const char* sb = reinterpret_cast<const char*>(smem) + slot_b + frag_offset(kLayB, wn * 128, ks, j);
        if (kLayB == kRowsByK) fb[set][j] = *reinterpret_cast<const bf16x8*>(sb);
        else fb[set][j] = read_transposed_fragment(sb);
    };
    auto read_frag_pair = [&](int set, uint32_t slot_a, uint32_t slot_b, int ks, int i) {
        read_frag_a(set, slot_a, ks, i);
        read_frag_b(set, slot_b, ks, i);
    };
    auto read_frags = [&](int set, uint32_t slot_a, uint32_t slot_b, int ks) {
#pragma unroll
        for (int i = 0; i < 4; ++i) read_frag_pair(set, slot_a, slot_b, ks, i);
    };
    // ring slots are named by their byte offset in LDS
    auto next_slot = [](uint32_t s) { return s + kTileBytes >= (uint32_t)kSmemBytes ? s + kTileBytes - kSmemBytes : s + kTileBytes; };

    if (step_begin < step_end) {
        // Operand tiles are numbered 2 s + o (o = 0 for A, 1 for B of step s) and tile t lives in ring
        // slot t mod 5.  Prologue: tiles 0..4 (steps 0, 1 and the A tile of step 2) are requested;
        // steps past the end re-request the last step's tiles, which nobody reads.
        const int last = step_end - 1;
        issue_loads(load_ctx(0, 0 * kTileBytes, step_begin), 0, 8);
        issue_loads(load_ctx(1, 1 * kTileBytes, step_begin), 0, 8);
        issue_loads(load_ctx(0, 2 * kTileBytes, min(step_begin + 1, last)), 0, 8);
        issue_loads(load_ctx(1, 3 * kTileBytes, min(step_begin + 1, last)), 0, 8);
        issue_loads(load_ctx(0, 4 * kTileBytes, min(step_begin + 2, last)), 0, 8);
        wait_direct_loads<3 * kLoadsPerTile>();
        __syncthreads();
        read_frags(0, 0 * kTileBytes, 1 * kTileBytes, 0);
        // One 64-wide step per trip.  `sa`, `sb` are the slots of this step's tiles; the next step's
        // are the two after them in the ring.  Fragment set 0 holds slice 0 of this step on entry and
        // slice 0 of the next step on exit.  The single barrier sits before the last slice: by then
        // every wavefront has issued all its reads of `sa`, `sb`, so both slots can be refilled, `sa`
        // with the B tile of step + 2 and `sb` with the A tile of step + 3.  At the barrier only the
        // newest tile (the A tile) may still be in flight.  The body is branch-free: near the end it
        // re-requests tiles that nobody reads.
        //
        // A wavefront issues in order and an MFMA keeps the matrix pipe busy for 32 cycles, so
        // whatever is issued between two MFMAs must fit in about 28 cycles or the pipe idles.  The
        // order is therefore fixed by hand, one memory instruction per gap: per MFMA row of a 16-wide
        // slice, one refill load (16 per step, one per row: issued together they would hold the
        // texture path for about 1000 cycles) and up to three fragment reads of the next slice.  The
        // last row has no reads, so that the reads of a slot have long landed when the barrier that
        // frees the slot waits for them; its gaps carry the scalar bookkeeping of the tile pointers.
        auto one_mfma = [&](int set, int i, int j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
        };
        // Reads of the next slice in the order its MFMAs need them: B0, B1, B2, A0, B3 for the first
        // row, then A1..A3.
        auto read_next = [&](int set, uint32_t rs_a, uint32_t rs_b, int ks, int n) {
            if (n < 3) read_frag_b(set, rs_b, ks, n);
            else if (n == 3) read_frag_a(set, rs_a, ks, 0);
            else if (n == 4) read_frag_b(set, rs_b, ks, 3);
            else if (n < 8) read_frag_a(set, rs_a, ks, n - 4);
        };
        // The 16 MFMAs of a slice walk the 4 x 4 tiles in serpentine order, so that consecutive
        // instructions always share one operand fragment.
        auto col = [](int g, int j) { return (g & 1) ? 3 - j : j; };
        auto slice = [&](int set, const LoadCtx& c, uint32_t half, uint32_t rs_a, uint32_t rs_b, int ks, auto hook) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                one_mfma(set, g, col(g, 0));
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(c, half * 4 + g, 1);
                __builtin_amdgcn_sched_barrier(0);
                one_mfma(set, g, col(g, 1));
                __builtin_amdgcn_sched_barrier(0);
                if (g < 3) read_next(set ^ 1, rs_a, rs_b, ks, 3 * g);
                __builtin_amdgcn_sched_barrier(0);
                one_mfma(set, g, col(g, 2));
                __builtin_amdgcn_sched_barrier(0);
                if (g < 3) read_next(set ^ 1, rs_a, rs_b, ks, 3 * g + 1);
                else hook(0);
                __builtin_amdgcn_sched_barrier(0);
                one_mfma(set, g, col(g, 3));
                __builtin_amdgcn_sched_barrier(0);
                if (g < 3) read_next(set ^ 1, rs_a, rs_b, ks, 3 * g + 2);
                else hook(1);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        uint32_t sa = 0;
        LoadCtx pend_b = load_ctx(0, 4 * kTileBytes, min(step_begin + 2, last));   // nothing pending yet: harmless re-request
        LoadCtx pend_a = pend_b;
        // tile streams: origin of the newest tile requested so far of each operand, and its step
        int at_a = min(step_begin + 2, last), at_b = min(step_begin + 1, last);
        const char* origin_a = tile_origin(0, at_a);
        const char* origin_b = tile_origin(1, at_b);
        auto no_hook = [](int) {};
        // The step counters run on past `last` (the origin then stands still, or lands once on the
        // start of the second segment, which is valid memory whether or not that segment is used).
        auto advance = [&](int operand) {
            if (operand == 0) {
                at_a += 1;
                origin_a += at_a <= last ? k_step_bytes[0] : (int64_t)0;
                origin_a = at_a == steps1 ? seg_origin[0][1] : origin_a;
            } else {
                at_b += 1;
                origin_b += at_b <= last ? k_step_bytes[1] : (int64_t)0;
                origin_b = at_b == steps1 ? seg_origin[1][1] : origin_b;
            }
        };
        // slots of this step's tiles and of the next step's; those of the step after are worked out in
        // otherwise empty gaps of the second slice
        uint32_t sb = next_slot(sa), na = next_slot(sb), nb = next_slot(na), after_a = 0, after_b = 0;
        auto rotate = [&](int half) {
            if (half == 0) after_a = next_slot(nb);
            else after_b = next_slot(after_a);
        };
        for (int step = step_begin; step < step_end; ++step) {
            slice(0, pend_b, 1, sa, sb, 1, no_hook);
            slice(1, pend_a, 0, sa, sb, 2, rotate);
            slice(0, pend_a, 1, sa, sb, 3, advance);
            wait_direct_loads<kLoadsPerTile>();
            __syncthreads();
            pend_b = load_ctx_at(1, sa, origin_b);   // tile 2 s + 5 -> slot of tile 2 s
            pend_a = load_ctx_at(0, sb, origin_a);   // tile 2 s + 6 -> slot of tile 2 s + 1
            slice(1, pend_b, 0, na, nb, 0, no_hook);
            sa = na;
            sb = nb;
            na = after_a;
            nb = after_b;
        }
        wait_direct_loads<0>();
        __syncthreads();
    }

    if (p.skip_if_empty && step_begin >= step_end && !runs_when_empty(epi, 0)) return;   // nothing to add (uniform over the workgroup)
    TileCoord tc{m0, n0, wm, wn, lane, split};
    epi(tc, acc, reinterpret_cast<char*>(smem));
}

// ---- epilogues -------------------------------------------------------------------------------

// 1 / (1 + e^-x) with the hardware exponential and reciprocal (about 1 ulp each; the results are
// rounded to bf16 afterwards).
__device__ inline float fast_sigmoid(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }

__device__ inline char* wave_stage(const TileCoord& tc, char* lds) {
    return lds + (tc.wm * 2 + tc.wn) * kWaveStageBytes;
}

// Writes bf16(acc[i][j]) for j in [j0, j0 + nj) of tile row i into a staging area whose rows are
// `stride` bytes apart: element (row, col) of the wavefront's sub-tile goes to
// stage + (row - row0) * stride + col_off * 2 + (32 (j - j0) + 8 q + 4 (lane >> 5)) * 2.
template <class F>
__device__ inline void stage_tile_row(char* stage, int stride, int lane, int local_row, int col_off, int nj, F value) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        if (jj >= nj) break;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = col_off + jj * 32 + 8 * q + 4 * (lane >> 5);
            *reinterpret_cast<bf16x4*>(stage + local_row * stride + col * 2) =
                to_bf16x4(value(jj, 4 * q), value(jj, 4 * q + 1), value(jj, 4 * q + 2), value(jj, 4 * q + 3));
        }
    }
}

// Staging area -> global memory, 16 bytes per lane: kRowBytes / 16 lanes cover one row, so a pass moves
// 1024 / kRowBytes rows and a 16-lane group writes whole 128-byte lines.  `dst` is this lane's address
// in row 0; rows at and beyond n_rows (wave-uniform) are not written.  Staging rows are 8-byte aligned
// only (their stride keeps the 8-byte writes of stage_tile_row conflict-free), hence two 8-byte reads.
template <int kRows, int kRowBytes>
__device__ inline void copy_rows_out(const char* st, int stride, char* dst, int64_t ld_bytes, int n_rows, int lane) {
    constexpr int kLanesPerRow = kRowBytes / 16, kRowsPerPass = 64 / kLanesPerRow;
    const char* src = st + (lane / kLanesPerRow) * stride + (lane % kLanesPerRow) * 16;
    char* out = dst + (lane / kLanesPerRow) * ld_bytes + (lane % kLanesPerRow) * 16;
    const int64_t out_step = kRowsPerPass * ld_bytes;
    if (n_rows >= kRows) {
#pragma unroll 8
        for (int pass = 0; pass < kRows / kRowsPerPass; ++pass) {
            const uint2 lo = *reinterpret_cast<const uint2*>(src), hi = *reinterpret_cast<const uint2*>(src + 8);
            *reinterpret_cast<uint4*>(out) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            src += kRowsPerPass * stride;
            out += out_step;
        }
    } else {
        int r = lane / kLanesPerRow;
        for (int pass = 0; pass < kRows / kRowsPerPass && pass * kRowsPerPass < n_rows; ++pass) {
            const uint2 lo = *reinterpret_cast<const uint2*>(src), hi = *reinterpret_cast<const uint2*>(src + 8);
            if (r < n_rows) *reinterpret_cast<uint4*>(out) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            src += kRowsPerPass * stride;
            out += out_step;
            r += kRowsPerPass;
        }
    }
}
// The same for fp32 rows that are added to what global memory holds (16 bytes = 4 floats per lane).
template <int kRows, int kRowBytes>
__device__ inline void add_rows_out(char* st, int stride, char* dst, int64_t ld_bytes, int lane) {
    constexpr int kLanesPerRow = kRowBytes / 16, kRowsPerPass = 64 / kLanesPerRow;
    char* src = st + (lane / kLanesPerRow) * stride + (lane % kLanesPerRow) * 16;
    char* out = dst + (lane / kLanesPerRow) * ld_bytes + (lane % kLanesPerRow) * 16;
    const int64_t out_step = kRowsPerPass * ld_bytes;
#pragma unroll 8
    for (int pass = 0; pass < kRows / kRowsPerPass; ++pass) {
        const f32x4 add = *reinterpret_cast<const f32x4*>(src);
        f32x4 cur = *reinterpret_cast<const f32x4*>(out);
        cur += add;
        *reinterpret_cast<f32x4*>(out) = cur;
        *reinterpret_cast<f32x4*>(src) = cur;      // the staging area now holds what was written (see staged_sum_of_squares)
        src += kRowsPerPass * stride;
        out += out_step;
    }
}
// Sum of the squares of the kRows fp32 rows in the staging area, this lane's share (the 16 bytes per pass that
// copy_rows_out / add_rows_out move), in fp64: squares of large fp32 values leave the fp32 range.
template <int kRows, int kRowBytes>
__device__ inline double staged_sum_of_squares(const char* st, int stride, int lane) {
    constexpr int kLanesPerRow = kRowBytes / 16, kRowsPerPass = 64 / kLanesPerRow;
    const char* src = st + (lane / kLanesPerRow) * stride + (lane % kLanesPerRow) * 16;
    double sq = 0.0;
#pragma unroll 1
    for (int pass = 0; pass < kRows / kRowsPerPass; ++pass) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(src);
        sq += (double)v[0] * (double)v[0] + (double)v[1] * (double)v[1] + (double)v[2] * (double)v[2] + (double)v[3] * (double)v[3];
        src += kRowsPerPass * stride;
    }
    return sq;
}
// Global memory -> staging area, the mirror image of copy_rows_out (all kRows rows), in two halves so
// that the loads can be in flight while other work runs: fetch_rows issues them into registers,
// stash_rows writes the registers to the staging area.
template <int kRows, int kRowBytes>
struct RowFetch {
    static constexpr int kLanesPerRow = kRowBytes / 16, kRowsPerPass = 64 / kLanesPerRow, kPasses = kRows / kRowsPerPass;
    uint4 r[kPasses];
    __device__ void fetch_rows(const char* src_row0, int64_t ld_bytes, int lane) {
        const char* in = src_row0 + (lane / kLanesPerRow) * ld_bytes + (lane % kLanesPerRow) * 16;
#pragma unroll
        for (int pass = 0; pass < kPasses; ++pass) r[pass] = *reinterpret_cast<const uint4*>(in + pass * kRowsPerPass * ld_bytes);
    }
    // The same with the rows given by number: rows[pass] is the row of a matrix (whose row 0, at this wavefront's
    // columns, is src_col0) that this lane fetches in that pass; a negative number stands for a row of zeros.
    __device__ void fetch_rows_at(const char* src_col0, int64_t ld_bytes, const int (&rows)[kPasses], int lane) {
        const char* in = src_col0 + (lane % kLanesPerRow) * 16;
#pragma unroll
        for (int pass = 0; pass < kPasses; ++pass)
            r[pass] = rows[pass] >= 0 ? *reinterpret_cast<const uint4*>(in + (int64_t)rows[pass] * ld_bytes)
                                      : make_uint4(0, 0, 0, 0);
    }
    __device__ void stash_rows(char* st, int stride, int lane) const {
        char* dst = st + (lane / kLanesPerRow) * stride + (lane % kLanesPerRow) * 16;
#pragma unroll
        for (int pass = 0; pass < kPasses; ++pass) {
            *reinterpret_cast<uint2*>(dst + pass * kRowsPerPass * stride) = make_uint2(r[pass].x, r[pass].y);
            *reinterpret_cast<uint2*>(dst + pass * kRowsPerPass * stride + 8) = make_uint2(r[pass].z, r[pass].w);
        }
    }
};
// copy_rows_out with the destination rows given by number (row i of the staging area goes to row rows[i] of the
// matrix whose row 0, at this wavefront's columns, is dst_col0; negative: not written).
template <int kRows, int kRowBytes>
__device__ inline void copy_rows_out_at(const char* st, int stride, char* dst_col0, int64_t ld_bytes, const int32_t* rows,
                                        int lane) {
    constexpr int kLanesPerRow = kRowBytes / 16, kRowsPerPass = 64 / kLanesPerRow;
    const char* src = st + (lane / kLanesPerRow) * stride + (lane % kLanesPerRow) * 16;
    char* out = dst_col0 + (lane % kLanesPerRow) * 16;
#pragma unroll 8
    for (int pass = 0; pass < kRows / kRowsPerPass; ++pass) {
        const int row = rows[lane / kLanesPerRow + pass * kRowsPerPass];
        const uint2 lo = *reinterpret_cast<const uint2*>(src), hi = *reinterpret_cast<const uint2*>(src + 8);
        if (row >= 0) *reinterpret_cast<uint4*>(out + (int64_t)row * ld_bytes) = make_uint4(lo.x, lo.y, hi.x, hi.y);
        src += kRowsPerPass * stride;
    }
}

// C (bf16, row-major) = acc; rows at and beyond row_limit are not written.
struct EpiStoreBf16 {
    bf16* C;
    int64_t ldc;
    int row_limit;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        constexpr int kStride = 264;                       // 128 bf16 + 8 bytes: conflict-free 8-byte accesses
        char* st = wave_stage(tc, lds);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            stage_tile_row(st, kStride, tc.lane, i * 32 + (tc.lane & 31), 0, 4,
                           [&](int j, int e) { return acc[i][j][e]; });
        __builtin_amdgcn_wave_barrier();
        const int row_base = tc.m0 + tc.wm * 128, col_base = tc.n0 + tc.wn * 128;
        copy_rows_out<128, 256>(st, kStride, reinterpret_cast<char*>(C + (int64_t)row_base * ldc + col_base), ldc * 2,
                                row_limit - row_base, tc.lane);
    }
};

// Rows of acc written to the rows of C (bf16, row-major) that row_idx names: row m of the product goes to row
// row_idx[m]; negative entries are not written.
struct EpiScatterBf16 {
    bf16* C;
    int64_t ldc;
    const int32_t* row_idx;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        constexpr int kStride = 264;
        char* st = wave_stage(tc, lds);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            stage_tile_row(st, kStride, tc.lane, i * 32 + (tc.lane & 31), 0, 4,
                           [&](int j, int e) { return acc[i][j][e]; });
        __builtin_amdgcn_wave_barrier();
        const int row_base = tc.m0 + tc.wm * 128, col_base = tc.n0 + tc.wn * 128;
        copy_rows_out_at<128, 256>(st, kStride, reinterpret_cast<char*>(C + col_base), ldc * 2, row_idx + row_base, tc.lane);
    }
};

// C (row-major) = acc as the sum of two bf16 matrices: hi = bf16(acc), lo = bf16(acc - hi), which together
// carry 16 bits of significand.  A following product that reads [hi | lo] as two reduction segments against the
// same second operand sees the value to about 2^-17 instead of 2^-9.  Rows at and beyond row_limit are not written.
struct EpiStoreBf16Split {
    bf16 *hi, *lo;
    int64_t ldc;
    int row_limit;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        constexpr int kStride = 520;                       // [hi 128 | lo 128] bf16 + 8 bytes
        char* st = wave_stage(tc, lds);
        const int col_base = tc.n0 + tc.wn * 128;
#pragma unroll
        for (int half = 0; half < 2; ++half) {             // 64 rows per pass
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int i = half * 2 + ii;
                char* row = st + (ii * 32 + (tc.lane & 31)) * kStride;
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float r[4];
                        bf16x4 h;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float x = acc[i][j][4 * q + t];
                            h[t] = (__bf16)x;
                            r[t] = x - (float)h[t];
                        }
                        char* at = row + (j * 32 + 8 * q + 4 * (tc.lane >> 5)) * 2;
                        *reinterpret_cast<bf16x4*>(at) = h;
                        *reinterpret_cast<bf16x4*>(at + 256) = to_bf16x4(r[0], r[1], r[2], r[3]);
                    }
            }
            __builtin_amdgcn_wave_barrier();
            const int row_base = tc.m0 + tc.wm * 128 + half * 64;
            const int64_t at = (int64_t)row_base * ldc + col_base;
            copy_rows_out<64, 256>(st, kStride, reinterpret_cast<char*>(hi + at), ldc * 2, row_limit - row_base, tc.lane);
            copy_rows_out<64, 256>(st + 256, kStride, reinterpret_cast<char*>(lo + at), ldc * 2, row_limit - row_base, tc.lane);
            __builtin_amdgcn_wave_barrier();
        }
    }
};

// Whether a row panel [row_begin, row_end) of a batch holds the batch's last live rows (panel 0 if there are none):
// the weight gradients that panel leaves are the final ones.
struct FinalPanel {
    const int32_t* n_kept;
    int max_chunks, A;
    int64_t row_begin, row_end;
    __device__ bool operator()() const {
        const int64_t rows = live_rows(n_kept, max_chunks, A);
        return rows <= row_end && (rows > row_begin || row_begin == 0);
    }
};

// C (fp32, row-major) = acc.  With a split reduction, part s goes to C + s * split_stride (its own
// M x N matrix; the caller sums the parts), so no atomics are needed and the sum is reproducible.
// accumulate: C += acc instead (a batch processed in row panels adds every panel's weight gradient).
// sumsq_parts (unsplit outputs with ldc = N only): on the final panel every wavefront also writes the sum of the
// squares of the values it leaves in C to sumsq_parts[4 * tile + wavefront] (for the gradient norm of the optimizer
// step, which then needs no pass of its own over the gradients).
struct EpiStoreF32 {
    float* C;
    int64_t ldc;
    int64_t split_stride;
    int accumulate;
    double* sumsq_parts;
    FinalPanel final_panel;
    __device__ bool runs_when_empty() const { return sumsq_parts != nullptr && final_panel(); }
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        float* const C = this->C + tc.split * split_stride;
        constexpr int kStride = 528;                       // 128 fp32 + 16 bytes: conflict-free 16-byte accesses
        char* st = wave_stage(tc, lds);
        const int col_base = tc.n0 + tc.wn * 128;
        const bool want_sq = sumsq_parts != nullptr && final_panel();
        double sq = 0.0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {                      // 32 rows per pass
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& a = acc[i][j];
                    f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                    *reinterpret_cast<f32x4*>(st + (tc.lane & 31) * kStride + (j * 32 + 8 * q + 4 * (tc.lane >> 5)) * 4) = v;
                }
            __builtin_amdgcn_wave_barrier();
            const int row_base = tc.m0 + tc.wm * 128 + i * 32;
            char* const dst = reinterpret_cast<char*>(C + (int64_t)row_base * ldc + col_base);
            if (accumulate) add_rows_out<32, 512>(st, kStride, dst, ldc * 4, tc.lane);
            else copy_rows_out<32, 512>(st, kStride, dst, ldc * 4, 32, tc.lane);
            if (want_sq) sq += staged_sum_of_squares<32, 512>(st, kStride, tc.lane);
            __builtin_amdgcn_wave_barrier();
        }
        if (want_sq) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
            const int tile = (tc.m0 / kTileM) * (int)(ldc / kTileN) + tc.n0 / kTileN;
            if (tc.lane == 0) sumsq_parts[tile * 4 + tc.wm * 2 + tc.wn] = sq;
        }
    }
};

// Gate/up projection with the activation fused: the B operand holds, per 128 packed rows, 64 gate
// columns followed by the 64 up columns of the same index range, so a wavefront's tiles j = 0, 1
// are u (gate) and j = 2, 3 the matching v (up).  Writes a = silu(u) * v (bf16, [M, ff]) and, for
// a backward pass to come, the two factors it will need, computed here where the sigmoid is at
// hand: fu = v * silu'(u) (so du = da * fu) and fv = silu(u) (so dv = da * fv).
// With kKeepLow the rounding remainder of a is written as well (a_lo = bf16(a - bf16(a))), for products
// that need the activation to more than bf16 precision (they read [a | a_lo] as two reduction segments).
template <bool kKeepFactors, bool kKeepLow = false>
struct EpiSwigluForward {
    bf16 *fu, *fv, *a, *a_lo;
    int64_t ld;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        // staged row: [a 64 | fu 64 | fv 64 | a_lo 64] bf16 (the parts that are kept) + 8 bytes
        constexpr int kLowAt = kKeepFactors ? 384 : 128;
        constexpr int kStride = 8 + 128 * (1 + (kKeepFactors ? 2 : 0) + (kKeepLow ? 1 : 0));
        char* st = wave_stage(tc, lds);
        const int col_base = ((tc.n0 + tc.wn * 128) / 128) * 64;
#pragma unroll
        for (int half = 0; half < 2; ++half) {             // 64 rows per pass
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int i = half * 2 + ii;
                char* row = st + (ii * 32 + (tc.lane & 31)) * kStride;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float av[4], fuv[4], fvv[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float x = acc[i][j][4 * q + t], y = acc[i][j + 2][4 * q + t];
                            const float sg = kKeepLow ? 1.f / (1.f + expf(-x)) : fast_sigmoid(x);   // full accuracy where it is kept
                            fvv[t] = x * sg;
                            av[t] = fvv[t] * y;
                            const float ys = y * sg;
                            fuv[t] = __builtin_fmaf(ys, x - fvv[t], ys);     // y sg (1 + x (1 - sg))
                        }
                        char* at = row + (j * 32 + 8 * q + 4 * (tc.lane >> 5)) * 2;
                        const bf16x4 a4 = to_bf16x4(av[0], av[1], av[2], av[3]);
                        *reinterpret_cast<bf16x4*>(at) = a4;
                        if (kKeepFactors) {
                            *reinterpret_cast<bf16x4*>(at + 128) = to_bf16x4(fuv[0], fuv[1], fuv[2], fuv[3]);
                            *reinterpret_cast<bf16x4*>(at + 256) = to_bf16x4(fvv[0], fvv[1], fvv[2], fvv[3]);
                        }
                        if (kKeepLow)
                            *reinterpret_cast<bf16x4*>(at + kLowAt) = to_bf16x4(av[0] - (float)a4[0], av[1] - (float)a4[1],
                                                                             av[2] - (float)a4[2], av[3] - (float)a4[3]);
                    }
            }
            __builtin_amdgcn_wave_barrier();
            const int row_base = tc.m0 + tc.wm * 128 + half * 64;
            const int64_t at = (int64_t)row_base * ld + col_base;     // 64 rows x 128 bytes of each output
            copy_rows_out<64, 128>(st, kStride, reinterpret_cast<char*>(a + at), ld * 2, 64, tc.lane);
            if (kKeepFactors) {
                copy_rows_out<64, 128>(st + 128, kStride, reinterpret_cast<char*>(fu + at), ld * 2, 64, tc.lane);
                copy_rows_out<64, 128>(st + 256, kStride, reinterpret_cast<char*>(fv + at), ld * 2, 64, tc.lane);
            }
            if (kKeepLow) copy_rows_out<64, 128>(st + kLowAt, kStride, reinterpret_cast<char*>(a_lo + at), ld * 2, 64, tc.lane);
            __builtin_amdgcn_wave_barrier();
        }
    }
};

// acc = da.  du = da * fu, dv = da * fv (bf16, [M, ff]; the factors are those written by the forward epilogue).
// kIndexed = false: in place, fu <- du, fv <- dv.  kIndexed = true: the rows of the product are a selection of the
// rows the forward pass ran over: product row m takes its factors from row row_idx[m] of fu, fv (negative: a row of
// zeros) and writes row m of du, dv (other buffers).  Works through the wavefront's 128 x 128 block in four passes of
// 32 rows; the rows of the next pass are fetched into registers while the current pass is computed.
template <bool kIndexed>
struct EpiSwigluBackward {
    bf16 *fu, *fv;
    int64_t ld;
    const int32_t* row_idx;
    bf16 *du, *dv;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        constexpr int kStride = 520;                       // [du 128 | dv 128] bf16 + 8 bytes
        char* st = wave_stage(tc, lds);
        const int row_base = tc.m0 + tc.wm * 128, col_base = tc.n0 + tc.wn * 128;
        const int64_t ld_bytes = ld * 2;
        const int64_t at = (kIndexed ? 0 : (int64_t)row_base * ld) + col_base;
        const char* const u0 = reinterpret_cast<const char*>(fu + at);
        const char* const v0 = reinterpret_cast<const char*>(fv + at);
        char* const du0 = reinterpret_cast<char*>((kIndexed ? du : fu) + (int64_t)row_base * ld + col_base);
        char* const dv0 = reinterpret_cast<char*>((kIndexed ? dv : fv) + (int64_t)row_base * ld + col_base);
        // the 128 row numbers of this wavefront's block, two per lane; a pass hands them to the lanes that fetch the rows
        int idx_lo = 0, idx_hi = 0;
        if (kIndexed) {
            idx_lo = row_idx[row_base + tc.lane];
            idx_hi = row_idx[row_base + 64 + tc.lane];
        }
        RowFetch<32, 256> ru, rv;
        auto fetch = [&](int pass) {
            if (kIndexed) {
                int rows[RowFetch<32, 256>::kPasses];
#pragma unroll
                for (int q = 0; q < RowFetch<32, 256>::kPasses; ++q)
                    rows[q] = __shfl(pass < 2 ? idx_lo : idx_hi,
                                     (pass & 1) * 32 + tc.lane / RowFetch<32, 256>::kLanesPerRow + q * RowFetch<32, 256>::kRowsPerPass, 64);
                ru.fetch_rows_at(u0, ld_bytes, rows, tc.lane);
                rv.fetch_rows_at(v0, ld_bytes, rows, tc.lane);
            } else {
                ru.fetch_rows(u0 + pass * 32 * ld_bytes, ld_bytes, tc.lane);
                rv.fetch_rows(v0 + pass * 32 * ld_bytes, ld_bytes, tc.lane);
            }
        };
        fetch(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {                      // 32 rows per pass
            ru.stash_rows(st, kStride, tc.lane);
            rv.stash_rows(st + 256, kStride, tc.lane);
            if (i < 3) fetch(i + 1);
            __builtin_amdgcn_wave_barrier();
            const int lr = tc.lane & 31;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = j * 32 + 8 * q + 4 * (tc.lane >> 5);
                    char* pu = st + lr * kStride + col * 2;
                    char* pv = pu + 256;
                    const bf16x4 u4 = *reinterpret_cast<const bf16x4*>(pu);
                    const bf16x4 v4 = *reinterpret_cast<const bf16x4*>(pv);
                    float gu[4], gv[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float g = acc[i][j][4 * q + t];
                        gu[t] = g * (float)u4[t];
                        gv[t] = g * (float)v4[t];
                    }
                    *reinterpret_cast<bf16x4*>(pu) = to_bf16x4(gu[0], gu[1], gu[2], gu[3]);
                    *reinterpret_cast<bf16x4*>(pv) = to_bf16x4(gv[0], gv[1], gv[2], gv[3]);
                }
            __builtin_amdgcn_wave_barrier();
            copy_rows_out<32, 256>(st, kStride, du0 + i * 32 * ld_bytes, ld_bytes, 32, tc.lane);
            copy_rows_out<32, 256>(st + 256, kStride, dv0 + i * 32 * ld_bytes, ld_bytes, 32, tc.lane);
            __builtin_amdgcn_wave_barrier();
        }
    }
};

// Logit projection (N = V = 256 = one tile, so a workgroup holds whole rows) with the loss fused:
// log-softmax at the target bin, row entropy, ratio, clipped surrogate and
// dz = coef * (onehot - softmax) + entropy_coef * scale * softmax * (log softmax + H) as bf16.
// With a per-chunk ratio the factor is not known yet: dz <- onehot - softmax, the entropy part goes
// to dz_extra, and the rows are scaled once the chunk ratios are known.
struct EpiLogitsLoss {
    const uint8_t* token;
    const float* logp_old;
    const float* adv_row;
    const int32_t* n_kept;
    int max_chunks, A;
    int row_offset;    // batch row of the panel's row 0 (the per-row arrays below are the panel's parts)
    LossOptions opt;
    bf16* dz;          // [M, 256] or nullptr
    bf16* dz_extra;    // [M, 256]: entropy part, per-chunk ratio only
    float* logp_out;   // may be nullptr
    RowOut out;
    __device__ void operator()(const TileCoord& tc, f32x16 (&acc)[4][4], char* lds) const {
        // exchange area (LDS, free after the main loop): [3 quantities][2 column halves][256 rows]
        float* ex_a = reinterpret_cast<float*>(lds);
        float* ex_b = ex_a + 512;
        float* ex_c = ex_b + 512;
        const int64_t rows_batch = live_rows(n_kept, max_chunks, A);
        const float scale = objective_scale(opt, rows_batch);
        const int64_t rows_live = rows_batch - row_offset;          // live rows of this panel (may be <= 0)
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

        float lse[4], ztok[4], ent[4];
        int tok[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tok[i] = token[tc.row(i)];
            float se = 0.f, sz = 0.f, zt = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = tc.col(j, q);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float z = acc[i][j][4 * q + t];
                        const float e = __expf(z - mx[i]);
                        se += e;
                        sz += e * z;
                        zt += (n + t == tok[i]) ? z : 0.f;
                    }
                }
            se += __shfl_xor(se, 32, 64);
            sz += __shfl_xor(sz, 32, 64);
            zt += __shfl_xor(zt, 32, 64);
            lse[i] = se;
            ent[i] = sz;
            ztok[i] = zt;
            if (tc.lane < 32) {
                ex_a[tc.wn * 256 + lrow_base + i * 32] = se;
                ex_b[tc.wn * 256 + lrow_base + i * 32] = zt;
                ex_c[tc.wn * 256 + lrow_base + i * 32] = sz;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int other = (tc.wn ^ 1) * 256 + lrow_base + i * 32;
            const float se = lse[i] + ex_a[other];
            lse[i] = mx[i] + __logf(se);
            ztok[i] += ex_b[other];
            ent[i] = lse[i] - (ent[i] + ex_c[other]) / se;      // H = -sum p log p
        }

#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tc.row(i);
            const bool live = m < rows_live;
            const float lp = ztok[i] - lse[i];
            const float w = (opt.chunk_weight && live) ? opt.chunk_weight[(m + row_offset) / A] : 1.f;
            const LossRow lr = loss_row(lp, logp_old[m], adv_row[m], w, opt, scale);
            if (tc.wn == 0 && tc.lane < 32) {
                out.dlogp[m] = lr.dlogp;
                out.entropy[m] = live ? ent[i] : 0.f;
                if (!opt.chunk_ratio) {
                    out.term[m] = live ? lr.term : 0.f;
                    out.ratio[m] = lr.ratio;
                    out.clipped[m] = lr.clipped;
                }
                if (logp_out && live) logp_out[m] = lp;
            }
            if (dz) {
                const float coef = opt.chunk_ratio ? (live ? 1.f : 0.f) : (live ? lr.coef : 0.f);
                const float ec = live ? opt.entropy_coef * scale : 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = tc.col(j, q);
                        float g[4], h[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float lpj = acc[i][j][4 * q + t] - lse[i];
                            const float pr = __expf(lpj);
                            g[t] = coef * (((n + t == tok[i]) ? 1.f : 0.f) - pr);
                            h[t] = ec * pr * (lpj + ent[i]);
                        }
                        if (opt.chunk_ratio) {
                            *reinterpret_cast<bf16x4*>(dz + (int64_t)m * 256 + n) = to_bf16x4(g[0], g[1], g[2], g[3]);
                            *reinterpret_cast<bf16x4*>(dz_extra + (int64_t)m * 256 + n) = to_bf16x4(h[0], h[1], h[2], h[3]);
                        } else {
                            *reinterpret_cast<bf16x4*>(dz + (int64_t)m * 256 + n) =
                                to_bf16x4(g[0] + h[0], g[1] + h[1], g[2] + h[2], g[3] + h[3]);
                        }
                    }
            }
        }
    }
};

template <int kLayA = kRowsByK, int kLayB = kRowsByK, class Epilogue>
inline void launch_gemm(const GemmProblem& p, const Epilogue& epi, hipStream_t s) {
    const unsigned grid = (unsigned)(p.M / kTileM) * (unsigned)(p.N / kTileN) * (unsigned)p.splits;
    gemm_bf16<Epilogue, kLayA, kLayB><<<grid, kGemmThreads, 0, s>>>(p, epi);
}

}  // namespace pcm
