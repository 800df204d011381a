// Stand-alone measurement aid (its own small library, not part of libpcm.so): the rate the matrix cores sustain on their own (no memory traffic) under the
// chip's power limit, which depends on the operand data: with all-zero operands the clock stays
// near its maximum, with random operands the power limit pulls it down by about a quarter.  The
// benchmark reports the GEMMs against this figure as well as against the nominal peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pcm_measure.h"

namespace pcm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ inline uint32_t lcg(uint32_t& s) {
    s = s * 1664525u + 1013904223u;
    return s;
}

// Roughly normal values (sum of four uniforms), or zeros.
__device__ inline __bf16 operand_value(uint32_t& s, int random) {
    if (!random) return (__bf16)0.f;
    float x = 0.f;
    for (int i = 0; i < 4; ++i) x += (float)(lcg(s) >> 8) * (1.f / 16777216.f) - 0.5f;
    return (__bf16)(x * 1.7f);
}

// One wavefront per SIMD, 16 independent accumulator tiles, operands held in registers.
__global__ __launch_bounds__(256, 1) void mfma_only(float* out, int iters, int random, long long* ticks) {
    uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    bf16x8 a[8], b[8];
    for (int r = 0; r < 8; ++r)
        for (int e = 0; e < 8; ++e) {
            a[r][e] = operand_value(s, random);
            b[r][e] = operand_value(s, random);
        }
    f32x16 acc[16];
    for (int t = 0; t < 16; ++t)
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 16; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t & 7], b[(t >> 2) + (t & 3)], acc[t], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float sum = 0.f;
    for (int t = 0; t < 16; ++t)
        for (int e = 0; e < 16; ++e) sum += acc[t][e];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;     // shader clock cycles
        ticks[1] = w1 - w0;     // constant-rate counter
    }
}

}  // namespace
}  // namespace pcm

using namespace pcm;

extern "C" int pcm_measure_mfma_rate(int random_operands, int milliseconds, double* tflops, double* clock_ghz) {
    if (!tflops || milliseconds < 1 || milliseconds > 2000) return PCM_EINVAL;
    int n_cu = 0, wall_khz = 0, device = 0;
    if (hipGetDevice(&device) != hipSuccess) return PCM_EHIP;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n_cu < 1) return PCM_EHIP;
    if (hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, device) != hipSuccess) wall_khz = 0;
    float* out = nullptr;
    long long* ticks = nullptr;
    if (hipMalloc(&out, (size_t)n_cu * 256 * sizeof(float)) != hipSuccess) return PCM_EHIP;
    if (hipMalloc(&ticks, 2 * sizeof(long long)) != hipSuccess) {
        (void)hipFree(out);
        return PCM_EHIP;
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = PCM_OK;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = PCM_EHIP;
    // 16 MFMAs of 32 cycles per trip: about 4700 trips per millisecond at 2.4 GHz
    const int iters = milliseconds * 4000;
    float ms = 0.f;
    long long h[2] = {0, 0};
    for (int rep = 0; rep < 2 && rc == PCM_OK; ++rep) {      // the first run settles the clock
        (void)hipEventRecord(e0, nullptr);
        mfma_only<<<n_cu, 256, 0, nullptr>>>(out, iters, random_operands, ticks);
        (void)hipEventRecord(e1, nullptr);
        if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
            hipMemcpy(h, ticks, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess)
            rc = PCM_EHIP;
    }
    if (rc == PCM_OK) {
        *tflops = (double)n_cu * 4 * iters * 16 * 32768.0 / ((double)ms * 1e9);
        if (clock_ghz) *clock_ghz = (h[1] > 0 && wall_khz > 0) ? (double)h[0] / (double)h[1] * wall_khz * 1e-6 : 0.0;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(ticks);
    (void)hipFree(out);
    return rc;
}
