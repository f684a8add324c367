// Register-resident fp32 MFMA loop: what the matrix cores of this GPU sustain
// with no memory traffic at all.  Used as a second denominator next to the
// published peak.  Prints one line per case: work-groups, ms, TFLOP/s.
#include <hip/hip_runtime.h>

#include <stdio.h>

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_loop(float *out, int iters, float a, float b)
{
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float x = a + threadIdx.x, y = b;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

#define CHECK(e) do { hipError_t err_ = (e); if (err_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #e, hipGetErrorString(err_)); return 1; } } while (0)

int main()
{
    const int wgs = 2048, iters = 4000;          // 8 work-groups per CU, 4 waves each
    float *d = nullptr;
    CHECK(hipMalloc(&d, (size_t)wgs * 256 * sizeof(float)));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const double flops = (double)wgs * 4 * iters * 32 * 4096.0;   // waves x iterations x MFMAs x 32*32*2*2
    hipLaunchKernelGGL(mfma_loop, dim3(wgs), dim3(256), 0, 0, d, 100, 1.f, 2.f);
    CHECK(hipDeviceSynchronize());
    float ms = 0.f;
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(mfma_loop, dim3(wgs), dim3(256), 0, 0, d, iters, 1.f, 2.f);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("burst      wgs=%d launches=1  ms=%.3f TFLOP/s=%.1f\n", wgs, ms, flops / ms / 1e9);
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(mfma_loop, dim3(wgs), dim3(256), 0, 0, d, iters, 1.f, 2.f);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("sustained  wgs=%d launches=10 ms=%.3f TFLOP/s=%.1f\n", wgs, ms, 10.0 * flops / ms / 1e9);
    CHECK(hipFree(d));
    return 0;
}
