// Internal helpers shared by the library's translation units (not part of the C boundary).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pcm.h"

namespace pcm {

constexpr int kWave = 64;  // gfx950 wavefront width

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace; every block is 256-byte aligned.
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align_up(count * sizeof(T), 256);
        return p;
    }
    size_t used() const { return off; }
};

inline bool workspace_ok(const void* ws, size_t have, size_t need) {
    if (need == 0) return true;
    return ws != nullptr && have >= need && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0;
}

// ---- stage timing ------------------------------------------------------------------------
enum Stage : int {
    ST_SCORE_PREPARE = 0,
    ST_SCORE_ACCUMULATE,
    ST_SCORE_FINALISE,
    ST_KEEP_PROBS,
    ST_SAMPLE_SCAN,
    ST_SAMPLE_COMPACT,
    ST_WEIGHT_LAYOUT,
    ST_GATHER,
    ST_GEMM_GATE_UP,
    ST_GEMM_DOWN,
    ST_GEMM_LOGITS_LOSS,
    ST_GEMM_DWO,
    ST_GEMM_DY,
    ST_GEMM_DWD,
    ST_GEMM_DA,
    ST_GEMM_DWG_DWU,
    ST_GEMM_DX,
    ST_REDUCE,
    ST_F32_FORWARD,
    ST_F32_LOSS,
    ST_F32_BACKWARD,
    ST_OPT_NORM,
    ST_OPT_ADAMW,
    ST_LABEL_PHASES,
    ST_LIVE_ROWS,
    ST_COUNT
};

bool profile_on();
void profile_begin(int stage, hipStream_t s);
void profile_end(int stage, hipStream_t s);

// Records a start/stop event pair around the launches made while it is alive.
struct StageTimer {
    int stage;
    hipStream_t s;
    bool on;
    StageTimer(int stage_, hipStream_t s_) : stage(stage_), s(s_), on(profile_on()) {
        if (on) profile_begin(stage, s);
    }
    ~StageTimer() {
        if (on) profile_end(stage, s);
    }
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? PCM_OK : PCM_EHIP; }

}  // namespace pcm
