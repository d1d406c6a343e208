// Sustained rate of the bf16 MFMA pipe alone: every wave keeps eight independent 32 x 32 x 16
// accumulations in flight out of registers, with no LDS or memory traffic.  The figure a contraction
// kernel can be held against at the clock the chip sustains under that load: with operands that are
// small integers it is the published peak, with random bf16 operands the power management lowers
// the clock and the rate with it.
#include <hip/hip_runtime.h>

#include "rapid.h"
#include "rapid_internal.h"

namespace rapid {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, unsigned seed, float* sink) {
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a, b;
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + seed;
#pragma unroll
    for (int e = 0; e < 8; ++e) {   // seed 0: a in {0, 1, 2, 3}, b = 1; else uniform in [-1, 1] in steps of 1e-3
        h = h * 1664525u + 1013904223u;
        const float x = seed ? (float)((int)((h >> 8) % 2001u) - 1000) * 1e-3f : (float)(threadIdx.x & 3);
        h = h * 1664525u + 1013904223u;
        const float y = seed ? (float)((int)((h >> 8) % 2001u) - 1000) * 1e-3f : 1.0f;
        a[e] = (__bf16)x;
        b[e] = (__bf16)y;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    if (sink) {   // never taken by the probe; keeps the accumulations alive
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][v];
        sink[blockIdx.x * 256u + threadIdx.x] = s;
    }
}

}  // namespace

int run_mfma_probe(int random_operands, int iters, int num_cu, double* tflops_out, double* ms_out, hipStream_t st) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return RAPID_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return RAPID_ERR_HIP;
    }
    const unsigned blocks = (unsigned)num_cu * 2;   // two workgroups of four waves per CU: two waves per SIMD
    const unsigned seed = random_operands ? 7u : 0u;
    mfma_probe_kernel<<<blocks, 256, 0, st>>>(iters / 10 + 1, seed, nullptr);   // warm-up, clocks ramp
    (void)hipEventRecord(e0, st);
    mfma_probe_kernel<<<blocks, 256, 0, st>>>(iters, seed, nullptr);
    (void)hipEventRecord(e1, st);
    int rc = RAPID_OK;
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = RAPID_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    const double flop = (double)blocks * 4.0 * iters * 8.0 * 2.0 * 32 * 32 * 16;
    if (ms_out) *ms_out = ms;
    if (tflops_out) *tflops_out = ms > 0.f ? flop / (ms * 1e-3) / 1e12 : 0.0;
    return RAPID_OK;
}

}  // namespace rapid
