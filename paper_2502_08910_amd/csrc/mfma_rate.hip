// Dense matrix-core throughput of the GPU as this library's kernels can see it:
// independent accumulation chains of one MFMA shape, no memory traffic.  Part of
// the measurement protocol (the prefill kernels are priced against the vendor
// peak and against this figure), not of the method.
#include "common.h"

namespace ihip {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// KIND 0: v_mfma_f32_32x32x16_bf16, 4 chains per wave; KIND 1: v_mfma_f32_16x16x32_bf16, 8 chains
template <int KIND>
__global__ __launch_bounds__(512) void mfma_rate_kernel(float *sink, int iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(float)((threadIdx.x - i) & 3);
    }
    float r = 0.f;
    if (KIND == 0) {
        f32x16 c[4] = {};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int u = 0; u < 4; ++u) c[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[u], 0, 0, 0);
        r = c[0][0] + c[1][1] + c[2][2] + c[3][3];
    } else {
        f32x4 c[8] = {};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int u = 0; u < 8; ++u) c[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[u], 0, 0, 0);
        for (int u = 0; u < 8; ++u) r += c[u][u & 3];
    }
    if (r == -1.0f) sink[threadIdx.x] = r;          // never true: keeps the chains alive
}

// returns the rate in TFLOP/s (2 flops per multiply-add), or a negative error
double measure_mfma_rate(int kind, int iters, float *sink, hipStream_t st)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1.0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1.0;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return -1.0;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -1.0; }
    const dim3 grid(cus * 2), block(512);            // 16 waves per compute unit: 4 per SIMD
    auto launch = [&] {
        if (kind == 0) hipLaunchKernelGGL(mfma_rate_kernel<0>, grid, block, 0, st, sink, iters);
        else hipLaunchKernelGGL(mfma_rate_kernel<1>, grid, block, 0, st, sink, iters);
    };
    launch();                                        // warm-up
    (void)hipEventRecord(e0, st);
    launch();
    (void)hipEventRecord(e1, st);
    float ms = 0.f;
    const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess &&
                    hipGetLastError() == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok || ms <= 0.f) return -1.0;
    const double per_wave = (kind == 0 ? 4.0 * 2 * 32 * 32 * 16 : 8.0 * 2 * 16 * 16 * 32) * iters;
    return per_wave * 8.0 * grid.x / (ms * 1e-3) / 1e12;
}

}  // namespace ihip
