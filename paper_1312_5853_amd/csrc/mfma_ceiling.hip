// Register-resident MFMA loops: what the matrix cores of this GPU sustain with
// no memory traffic at all, fp32 (v_mfma_f32_32x32x2_f32) and bf16
// (v_mfma_f32_32x32x16_bf16; with operands that never change, and with eight
// sets of pseudo-random operands cycled, which is what real data costs in
// power and therefore in clock).  bench.py reports them as second denominators
// next to the published peaks.  It also measures what one CU moves per clock
// through its LDS (ds_read_b128, ds_write_b128 from registers) and through the
// vector memory path (16-byte loads of cache-resident data into registers, and
// straight into LDS): the three rates that decide how the bf16 kernels stage
// their operands.  Prints one line per case.
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

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ unsigned mix(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }
// a pair of bf16 values with magnitudes in [1, 2) and random signs and fractions (sums stay finite)
__device__ unsigned bf16_pair(unsigned s) { return 0x3F803F80u | (mix(s) & 0x807F807Fu); }

template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_bf16_loop(float *out, int iters)
{
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    u32x4 a[8], b[8];
    for (int s = 0; s < 8; ++s)
        for (int k = 0; k < 4; ++k) {
            a[s][k] = RANDOM ? bf16_pair(threadIdx.x * 131 + s * 17 + k) : 0x3F803F80u;
            b[s][k] = RANDOM ? bf16_pair(threadIdx.x * 257 + s * 29 + k + 99) : 0x3F803F80u;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(u + i) & 7]),
                                                                 __builtin_bit_cast(bf16x8, b[(u * 3 + i) & 7]),
                                                                 acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// --- LDS and vector-memory rates per CU (512 work-groups of 256 threads, eight independent accesses per iteration)
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int MODE>   // 0 ds_read_b128, 1 ds_write_b128, 2 global_load_dwordx4, 3 global_load_lds_dwordx4
__global__ __launch_bounds__(256) void rate_kernel(const float *src, float *out, int iters)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 8192; i += 256) sm[i] = (float)i;
    __syncthreads();
    // LDS: the fragment pattern of the kernels (row lane % 32 of 36-word rows, 16-byte piece lane / 32): conflict-free
    const unsigned laddr = (unsigned)(size_t)sm + (unsigned)((wave * 32 * 36 + (lane & 31) * 36 + (lane >> 5) * 4) * 4);
    // memory: each work-group streams its own 64 KB window (stays in the caches), 1 KB per wavefront access
    const char *g = reinterpret_cast<const char *>(src) + (size_t)(blockIdx.x & 63) * 65536 + wave * 16384 + lane * 16;
    const unsigned dma_base = (unsigned)(size_t)sm + (unsigned)(wave * 8192);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    f32x4 w = {1.f, 2.f, 3.f, (float)tid};
    for (int it = 0; it < iters; ++it) {
        f32x4 v[8];
        if (MODE == 0) {
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_read_b128 %0, %1" : "=v"(v[u]) : "v"(laddr));
            asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        } else if (MODE == 1) {
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_write_b128 %0, %1" :: "v"(laddr), "v"(w) : "memory");
        } else if (MODE == 2) {
            const char *gi = g + (it & 1) * 8192;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v[u]) : "v"(gi + u * 1024));
            asm volatile("s_waitcnt vmcnt(0)");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        } else {
            const char *gi = g + (it & 1) * 8192;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(dma_base + u * 1024), "v"(gi + u * 1024));
            asm volatile("s_waitcnt vmcnt(0)");
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)");
    __syncthreads();
    out[blockIdx.x * 256 + tid] = acc[0] + acc[1] + acc[2] + acc[3] + sm[tid];
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
    // bf16: 512 work-groups (two waves per SIMD), 0.1 s each
    const int bwgs = 512, biters = 10000;
    const double bflops = (double)bwgs * 4 * biters * 32 * 32768.0;      // waves x iterations x MFMAs x 32*32*16*2
    for (int rnd = 0; rnd < 2; ++rnd) {
        if (rnd) hipLaunchKernelGGL(mfma_bf16_loop<true>, dim3(bwgs), dim3(256), 0, 0, d, 100);
        else hipLaunchKernelGGL(mfma_bf16_loop<false>, dim3(bwgs), dim3(256), 0, 0, d, 100);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        if (rnd) hipLaunchKernelGGL(mfma_bf16_loop<true>, dim3(bwgs), dim3(256), 0, 0, d, biters);
        else hipLaunchKernelGGL(mfma_bf16_loop<false>, dim3(bwgs), dim3(256), 0, 0, d, biters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        printf("%s wgs=%d ms=%.3f TFLOP/s=%.1f\n", rnd ? "bf16_sustained_random_operands  " : "bf16_sustained_constant_operands",
               bwgs, ms, bflops / ms / 1e9);
    }
    // bytes per clock and CU (at the 2.4 GHz peak clock) of LDS reads, LDS writes from registers, cache-resident
    // 16-byte loads into registers, and the same loads straight into LDS
    {
        float *src = nullptr;
        CHECK(hipMalloc(&src, 64 * 65536));
        CHECK(hipMemset(src, 0, 64 * 65536));
        const int rwgs = 512, riters = 4000;
        const char *names[4] = {"lds_read_b128 ", "lds_write_b128", "load_dwordx4  ", "load_lds_dwordx4"};
        for (int mode = 0; mode < 4; ++mode) {
            for (int rep = 0; rep < 2; ++rep) {        // first launch warms up
                const int it = rep ? riters : 50;
                CHECK(hipEventRecord(e0));
                if (mode == 0) hipLaunchKernelGGL(rate_kernel<0>, dim3(rwgs), dim3(256), 32768, 0, src, d, it);
                else if (mode == 1) hipLaunchKernelGGL(rate_kernel<1>, dim3(rwgs), dim3(256), 32768, 0, src, d, it);
                else if (mode == 2) hipLaunchKernelGGL(rate_kernel<2>, dim3(rwgs), dim3(256), 32768, 0, src, d, it);
                else hipLaunchKernelGGL(rate_kernel<3>, dim3(rwgs), dim3(256), 32768, 0, src, d, it);
                CHECK(hipEventRecord(e1));
                CHECK(hipEventSynchronize(e1));
            }
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            const double bytes_per_cu = (double)rwgs / 256 * 4 * riters * 8 * 1024.0;
            printf("rate_%s bytes_per_clk_per_cu=%.1f (clocks per wavefront access: %.1f)\n", names[mode],
                   bytes_per_cu / (ms * 1e-3 * 2.4e9), 1024.0 * (ms * 1e-3 * 2.4e9) / bytes_per_cu);
        }
        CHECK(hipFree(src));
    }
    CHECK(hipFree(d));
    return 0;
}
