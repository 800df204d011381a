// Version/status strings and the optional stage timer (host code only).
#include <mutex>
#include <vector>

#include "common.h"
#include "pcm_measure.h"

namespace pcm {
namespace {

const char* const kStageNames[ST_COUNT] = {
    "score_prepare",   "score_accumulate", "score_finalise", "keep_probs",  "sample_scan",
    "sample_compact",  "weight_layout",    "gather",         "gemm_gate_up", "gemm_down",
    "gemm_logits_loss", "gemm_dWo",        "gemm_dy",        "gemm_dWd",    "gemm_da",
    "gemm_dWg_dWu",    "gemm_dX",          "reduce",         "f32_forward", "f32_loss",
    "f32_backward",    "opt_grad_norm",    "opt_adamw",
    "label_phases",    "live_rows"};

struct Pending {
    int stage;
    hipEvent_t start, stop;
};

struct Profiler {
    std::mutex mu;
    bool on = false;
    std::vector<hipEvent_t> pool;
    std::vector<Pending> pending;
    hipEvent_t open_start[ST_COUNT] = {};
    double total_ms[ST_COUNT] = {};
    int64_t launches[ST_COUNT] = {};

    hipEvent_t get() {
        if (!pool.empty()) {
            hipEvent_t e = pool.back();
            pool.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

Profiler& prof() {
    static Profiler p;
    return p;
}

}  // namespace

bool profile_on() { return prof().on; }

void profile_begin(int stage, hipStream_t s) {
    Profiler& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    hipEvent_t e = p.get();
    if (!e) return;
    (void)hipEventRecord(e, s);
    p.open_start[stage] = e;
}

void profile_end(int stage, hipStream_t s) {
    Profiler& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    hipEvent_t st = p.open_start[stage];
    if (!st) return;
    hipEvent_t e = p.get();
    if (!e) return;
    (void)hipEventRecord(e, s);
    p.pending.push_back({stage, st, e});
    p.open_start[stage] = nullptr;
}

}  // namespace pcm

using namespace pcm;

extern "C" const char* pcm_version(void) { return "pcm-gfx950 0.1"; }

extern "C" const char* pcm_status_string(int status) {
    switch (status) {
        case PCM_OK: return "ok";
        case PCM_EINVAL: return "invalid argument";
        case PCM_EWORKSPACE: return "workspace missing, misaligned or too small";
        case PCM_EHIP: return "HIP error";
        case PCM_EUNSUPPORTED: return "unsupported shape or dtype";
        default: return "unknown status";
    }
}

extern "C" int pcm_profile_enable(int on) {
    Profiler& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    if (on && !p.on) {
        for (int i = 0; i < ST_COUNT; ++i) {
            p.total_ms[i] = 0;
            p.launches[i] = 0;
        }
    }
    p.on = on != 0;
    return PCM_OK;
}

extern "C" int pcm_profile_stage_count(void) { return ST_COUNT; }

extern "C" const char* pcm_profile_stage_name(int stage) {
    return (stage >= 0 && stage < ST_COUNT) ? kStageNames[stage] : nullptr;
}

extern "C" int pcm_profile_collect(double* total_ms, int64_t* launches) {
    Profiler& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    int rc = PCM_OK;
    for (const Pending& q : p.pending) {
        if (hipEventSynchronize(q.stop) != hipSuccess) rc = PCM_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, q.start, q.stop) == hipSuccess) {
            p.total_ms[q.stage] += ms;
            p.launches[q.stage] += 1;
        } else {
            rc = PCM_EHIP;
        }
        p.pool.push_back(q.start);
        p.pool.push_back(q.stop);
    }
    p.pending.clear();
    for (int i = 0; i < ST_COUNT; ++i) {
        if (total_ms) total_ms[i] = p.total_ms[i];
        if (launches) launches[i] = p.launches[i];
    }
    return rc;
}
