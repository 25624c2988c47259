// Stand-alone probe of the two rates the fill kernel's roofline is built on: plain (non-packed)
// vector ALU operations and LDS reads of consecutive dwords, per compute unit and clock.
// Every access is in bounds and every loop has a fixed trip count.  Build: see build.py; run:
//     ./peaks_probe
#include <hip/hip_runtime.h>

#include <stdio.h>
#include <stdlib.h>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
            exit(1);                                                                  \
        }                                                                             \
    } while (0)

constexpr int kIters = 4096;

// fp32 add + min on 8 independent chains per lane (the D-record update).
__global__ __launch_bounds__(256) void valu_add_min(float *out, float c, int iters)
{
    float a[8], b[8];
    for (int j = 0; j < 8; ++j) {
        a[j] = threadIdx.x * 0.5f + j;
        b[j] = 1e30f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            a[j] = a[j] + c;
            b[j] = fminf(b[j], a[j]);
        }
    }
    float s = 0;
    for (int j = 0; j < 8; ++j)
        s += b[j] + a[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// fp32 add + compare + two selects (the level-tracking update as Alg. 1 writes it).
__global__ __launch_bounds__(256) void valu_add_cmp_sel(float *out, float c, int iters)
{
    float a[8], b[8];
    int g[8];
    for (int j = 0; j < 8; ++j) {
        a[j] = threadIdx.x * 0.5f + j;
        b[j] = 1e30f;
        g[j] = 0;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            a[j] = a[j] + c;
            const bool lt = a[j] < b[j];
            b[j] = lt ? a[j] : b[j];
            g[j] = lt ? i : g[j];
        }
    }
    float s = 0;
    for (int j = 0; j < 8; ++j)
        s += b[j] + a[j] + g[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Eight LDS reads of width sizeof(T) per iteration at immediate offsets; consecutive lanes read
// consecutive elements, the base moves by `step` dwords per iteration inside the buffer.
template <typename T>
__global__ __launch_bounds__(256) void lds_read(int *out, int step, int iters, int words)
{
    extern __shared__ int lds[];
    for (int i = threadIdx.x; i < words; i += blockDim.x)
        lds[i] = i;
    __syncthreads();
    constexpr int W = sizeof(T) / 4;
    const int mask = words / 2 - 1;   // bases stay in the lower half, reads reach + 8*64*W words
    int idx = (threadIdx.x * W) & mask;
    int acc = 0;
    for (int i = 0; i < iters; ++i) {
        const T *p = reinterpret_cast<const T *>(lds + idx);
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            const T x = p[j * 64], y = p[(j + 1) * 64];
            const int *xi = reinterpret_cast<const int *>(&x);
            const int *yi = reinterpret_cast<const int *>(&y);
#pragma unroll
            for (int w = 0; w < W; ++w)
                acc = acc + xi[w] + yi[w];
        }
        idx = (idx + step) & mask;
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

template <typename F>
float time_ms(F launch, int reps)
{
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    for (int i = 0; i < 200; ++i)     // some tens of milliseconds: the core clock settles
        launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i)
        launch();
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms;
    CHECK(hipEventElapsedTime(&ms, a, b));
    return ms / reps;
}

int main()
{
    hipDeviceProp_t p;
    CHECK(hipGetDeviceProperties(&p, 0));
    const int cus = p.multiProcessorCount;
    const double clk = p.clockRate * 1e3;
    printf("device %s, %d CUs, %.0f MHz, %zu B LDS per workgroup\n", p.gcnArchName, cus,
           clk / 1e6, p.sharedMemPerBlock);
    const int blocks = cus * 8, threads = 256;
    float *out;
    CHECK(hipMalloc(&out, sizeof(float) * blocks * threads));

    float ms = time_ms([&] { hipLaunchKernelGGL(valu_add_min, dim3(blocks), dim3(threads), 0, 0,
                                                out, 1.0f, kIters); }, 20);
    double ops = (double)blocks * threads * kIters * 16;
    printf("VALU add+min        : %.3f ms  %.2f Tlane-op/s  %.1f lane-ops/clk/CU\n", ms,
           ops / ms / 1e9, ops / (ms * 1e-3) / clk / cus);
    ms = time_ms([&] { hipLaunchKernelGGL(valu_add_cmp_sel, dim3(blocks), dim3(threads), 0, 0,
                                          out, 1.0f, kIters); }, 20);
    ops = (double)blocks * threads * kIters * 32;
    printf("VALU add+cmp+2 sel  : %.3f ms  %.2f Tlane-op/s  %.1f lane-ops/clk/CU\n", ms,
           ops / ms / 1e9, ops / (ms * 1e-3) / clk / cus);

    const int words = 8192;    // 32 KB per workgroup, four workgroups (16 waves) per CU
    const int nb = cus * 4;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(lds_read<int>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, words * 4));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(lds_read<int2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, words * 4));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(lds_read<int4>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, words * 4));
    for (int step : {64, 65, 1}) {
        ms = time_ms([&] { hipLaunchKernelGGL(lds_read<int>, dim3(nb), dim3(threads), words * 4, 0,
                                              (int *)out, step, kIters, words); }, 10);
        const double bytes = (double)nb * threads * kIters * 8 * 4;
        printf("LDS 32-bit reads, base step %2d dwords : %.3f ms  %.1f TB/s  %.1f B/clk/CU\n", step,
               ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / clk / cus);
    }
    for (int step : {64, 2}) {
        ms = time_ms([&] { hipLaunchKernelGGL(lds_read<int2>, dim3(nb), dim3(threads), words * 4, 0,
                                              (int *)out, step, kIters / 2, words); }, 10);
        const double bytes = (double)nb * threads * (kIters / 2) * 8 * 8;
        printf("LDS 64-bit reads, base step %2d dwords : %.3f ms  %.1f TB/s  %.1f B/clk/CU\n", step,
               ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / clk / cus);
    }
    for (int step : {64, 4}) {
        ms = time_ms([&] { hipLaunchKernelGGL(lds_read<int4>, dim3(nb), dim3(threads), words * 4, 0,
                                              (int *)out, step, kIters / 4, words); }, 10);
        const double bytes = (double)nb * threads * (kIters / 4) * 8 * 16;
        printf("LDS 128-bit reads, base step %2d dwords: %.3f ms  %.1f TB/s  %.1f B/clk/CU\n", step,
               ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / clk / cus);
    }
    CHECK(hipFree(out));
    return 0;
}
