// Optimizer step that follows the actor gradients (App. D, training details): global-norm gradient
// clipping, then AdamW on fp32 master weights, with an optional bf16 copy of the new weights for
// the next forward pass.  Pure streaming work: every gradient is read twice (norm, update) and
// every state element once.
//
//   pass 1  sumsq_chunks   one fp64 partial sum of g^2 per 4096-element chunk
//   pass 2  finish_norm    one workgroup adds the partials in a fixed order -> norm, clip factor
//   pass 3  adamw_chunks   m, v, theta updated in place, low-precision copy written
//
// The tensors are addressed as one list of chunks, so the whole head is one launch per pass.
#include "common.h"

namespace pcm {
namespace {

constexpr int kMaxTensors = PCM_MAX_OPT_TENSORS;
constexpr int kChunk = 4096;          // elements per workgroup: 256 lanes x 4 float4
constexpr int kThreads = 256;

struct TensorList {
    const float* grad[kMaxTensors];
    float* weight[kMaxTensors];
    float* m[kMaxTensors];
    float* v[kMaxTensors];
    uint16_t* lowp[kMaxTensors];      // bf16 copy of the weights, or null
    int64_t numel[kMaxTensors];
    int64_t first_chunk[kMaxTensors + 1];
    int n;
};

struct NormResult {
    double sumsq;
    float norm, scale;
};

__device__ inline void locate(const TensorList& tl, int64_t chunk, int& tensor, int64_t& begin) {
    int t = 0;
    while (t + 1 < tl.n && chunk >= tl.first_chunk[t + 1]) ++t;
    tensor = t;
    begin = (chunk - tl.first_chunk[t]) * kChunk;
}

__device__ inline double block_sum(double x, double* lds) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) total += lds[w];
    return total;   // valid in thread 0
}

__global__ __launch_bounds__(kThreads) void sumsq_chunks(TensorList tl, double* partial) {
    __shared__ double lds[kThreads / 64];
    int t;
    int64_t begin;
    locate(tl, blockIdx.x, t, begin);
    const float* g = tl.grad[t];
    const int64_t n = tl.numel[t];
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t i = begin + ((int64_t)r * kThreads + threadIdx.x) * 4;
        if (i + 3 < n) {
            const float4 x = *reinterpret_cast<const float4*>(g + i);
            acc += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        } else {
            for (int64_t j = i; j < n; ++j) acc += g[j] * g[j];
        }
    }
    const double total = block_sum((double)acc, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(1024) void finish_norm(const double* partial, int64_t n_chunks, double max_norm,
                                                    double clip_eps, NormResult* result, float* norm_out) {
    __shared__ double lds[16];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_chunks; i += blockDim.x) acc += partial[i];
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const double norm = sqrt(total);
        const double scale = fmin(1.0, max_norm / (norm + clip_eps));
        result->sumsq = total;
        result->norm = (float)norm;
        result->scale = (float)scale;
        if (norm_out) *norm_out = (float)norm;
    }
}

struct AdamConst {
    float beta1, beta2, one_minus_beta1, one_minus_beta2;
    float decay;            // 1 - lr * weight_decay
    float step_size;        // lr / (1 - beta1^t)
    float inv_sqrt_bc2;     // 1 / sqrt(1 - beta2^t)
    float eps;
};

__device__ inline uint16_t to_bf16_bits(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

__device__ inline float adam_one(float g, float& m, float& v, float w, const AdamConst& c) {
    m = c.beta1 * m + c.one_minus_beta1 * g;
    v = c.beta2 * v + c.one_minus_beta2 * (g * g);
    const float denom = sqrtf(v) * c.inv_sqrt_bc2 + c.eps;
    return w * c.decay - c.step_size * (m / denom);
}

__global__ __launch_bounds__(kThreads) void adamw_chunks(TensorList tl, const NormResult* result, AdamConst c) {
    int t;
    int64_t begin;
    locate(tl, blockIdx.x, t, begin);
    const float* g = tl.grad[t];
    float* w = tl.weight[t];
    float* m = tl.m[t];
    float* v = tl.v[t];
    uint16_t* lp = tl.lowp[t];
    const int64_t n = tl.numel[t];
    const float scale = result->scale;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t i = begin + ((int64_t)r * kThreads + threadIdx.x) * 4;
        if (i + 3 < n) {
            const float4 g4 = *reinterpret_cast<const float4*>(g + i);
            float4 m4 = *reinterpret_cast<const float4*>(m + i);
            float4 v4 = *reinterpret_cast<const float4*>(v + i);
            float4 w4 = *reinterpret_cast<const float4*>(w + i);
            w4.x = adam_one(g4.x * scale, m4.x, v4.x, w4.x, c);
            w4.y = adam_one(g4.y * scale, m4.y, v4.y, w4.y, c);
            w4.z = adam_one(g4.z * scale, m4.z, v4.z, w4.z, c);
            w4.w = adam_one(g4.w * scale, m4.w, v4.w, w4.w, c);
            *reinterpret_cast<float4*>(m + i) = m4;
            *reinterpret_cast<float4*>(v + i) = v4;
            *reinterpret_cast<float4*>(w + i) = w4;
            if (lp) {
                ushort4 b;
                b.x = to_bf16_bits(w4.x); b.y = to_bf16_bits(w4.y); b.z = to_bf16_bits(w4.z); b.w = to_bf16_bits(w4.w);
                *reinterpret_cast<ushort4*>(lp + i) = b;
            }
        } else {
            for (int64_t j = i; j < n; ++j) {
                float mj = m[j], vj = v[j];
                const float wj = adam_one(g[j] * scale, mj, vj, w[j], c);
                m[j] = mj; v[j] = vj; w[j] = wj;
                if (lp) lp[j] = to_bf16_bits(wj);
            }
        }
    }
}

int64_t count_chunks(int n, const int64_t* numel) {
    int64_t c = 0;
    for (int i = 0; i < n; ++i) c += (numel[i] + kChunk - 1) / kChunk;
    return c;
}

struct OptWorkspace {
    double* partial;
    NormResult* result;
    size_t bytes;
};

OptWorkspace carve(void* ws, int64_t n_chunks) {
    Carver c(ws);
    OptWorkspace w{};
    w.partial = c.take<double>((size_t)n_chunks);
    w.result = c.take<NormResult>(1);
    w.bytes = c.used();
    return w;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" {

PCM_API size_t pcm_adamw_clip_step_workspace_bytes(int n_tensors, const int64_t* numel) {
    if (n_tensors < 1 || n_tensors > kMaxTensors || numel == nullptr) return 0;
    for (int i = 0; i < n_tensors; ++i)
        if (numel[i] < 1) return 0;
    return carve(nullptr, count_chunks(n_tensors, numel)).bytes;
}

PCM_API int pcm_adamw_clip_step_ex(int n_tensors, const int64_t* numel, const float* const* grads, float* const* weights,
                                   float* const* m, float* const* v, void* const* weights_bf16, int64_t step, double lr,
                                   double beta1, double beta2, double eps, double weight_decay, double max_grad_norm,
                                   const double* grad_sumsq, float* grad_norm_out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    if (reinterpret_cast<uintptr_t>(grad_sumsq) & 7u) return PCM_EINVAL;
    if (n_tensors < 1 || n_tensors > kMaxTensors || !numel || !grads || !weights || !m || !v) return PCM_EINVAL;
    if (step < 1 || !(lr >= 0.0) || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || !(eps > 0.0) ||
        !(weight_decay >= 0.0) || !(max_grad_norm > 0.0))
        return PCM_EINVAL;
    TensorList tl{};
    tl.n = n_tensors;
    int64_t chunks = 0;
    for (int i = 0; i < n_tensors; ++i) {
        if (numel[i] < 1 || !grads[i] || !weights[i] || !m[i] || !v[i]) return PCM_EINVAL;
        void* lp = weights_bf16 ? weights_bf16[i] : nullptr;
        if (!aligned16(grads[i]) || !aligned16(weights[i]) || !aligned16(m[i]) || !aligned16(v[i]) ||
            (reinterpret_cast<uintptr_t>(lp) & 7u) != 0)
            return PCM_EINVAL;
        tl.grad[i] = grads[i]; tl.weight[i] = weights[i]; tl.m[i] = m[i]; tl.v[i] = v[i];
        tl.lowp[i] = static_cast<uint16_t*>(lp);
        tl.numel[i] = numel[i];
        tl.first_chunk[i] = chunks;
        chunks += (numel[i] + kChunk - 1) / kChunk;
    }
    tl.first_chunk[n_tensors] = chunks;
    if (chunks > 0x7fffffffLL) return PCM_EUNSUPPORTED;
    OptWorkspace w = carve(workspace, chunks);
    if (!workspace_ok(workspace, workspace_bytes, w.bytes)) return PCM_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    AdamConst c;
    c.beta1 = (float)beta1; c.beta2 = (float)beta2;
    c.one_minus_beta1 = (float)(1.0 - beta1); c.one_minus_beta2 = (float)(1.0 - beta2);
    c.decay = (float)(1.0 - lr * weight_decay);
    c.step_size = (float)(lr / (1.0 - pow(beta1, (double)step)));
    c.inv_sqrt_bc2 = (float)(1.0 / sqrt(1.0 - pow(beta2, (double)step)));
    c.eps = (float)eps;
    {
        StageTimer t(ST_OPT_NORM, s);
        if (grad_sumsq != nullptr) {      // the sum of squares is given: one "partial"
            finish_norm<<<1, 1024, 0, s>>>(grad_sumsq, 1, max_grad_norm, 1e-6, w.result, grad_norm_out);
        } else {
            sumsq_chunks<<<(unsigned)chunks, kThreads, 0, s>>>(tl, w.partial);
            finish_norm<<<1, 1024, 0, s>>>(w.partial, chunks, max_grad_norm, 1e-6, w.result, grad_norm_out);
        }
    }
    {
        StageTimer t(ST_OPT_ADAMW, s);
        adamw_chunks<<<(unsigned)chunks, kThreads, 0, s>>>(tl, w.result, c);
    }
    return launch_status();
}

PCM_API int pcm_adamw_clip_step(int n_tensors, const int64_t* numel, const float* const* grads, float* const* weights,
                                float* const* m, float* const* v, void* const* weights_bf16, int64_t step, double lr,
                                double beta1, double beta2, double eps, double weight_decay, double max_grad_norm,
                                float* grad_norm_out, void* workspace, size_t workspace_bytes, void* stream) {
    return pcm_adamw_clip_step_ex(n_tensors, numel, grads, weights, m, v, weights_bf16, step, lr, beta1, beta2, eps,
                                  weight_decay, max_grad_norm, nullptr, grad_norm_out, workspace, workspace_bytes, stream);
}

}  // extern "C"
