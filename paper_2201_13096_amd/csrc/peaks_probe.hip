// Stand-alone probe of the rates the fill kernel's roofline is built on, per compute unit and
// clock: plain (non-packed) vector ALU instructions in the mixes the fill issues, and LDS reads of
// consecutive elements at the widths it uses.  bench.py runs it as a child process before it
// touches the GPU itself and puts the figures next to the nominal peaks in its output line.
// Every access is in bounds and every loop has a fixed trip count.  Prints one JSON object.
//
// The ALU loops are written with inline assembly, one statement per instruction, so the number
// of issued vector instructions is the number written here (the loop counter and branch are
// scalar instructions): "lane_ops" below counts issued VALU instructions x 64 lanes, never
// source-level operations.
#include <hip/hip_runtime.h>

#include <stdio.h>
#include <stdlib.h>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                                  \
        }                                                                             \
    } while (0)

constexpr int kIters = 4096;
constexpr int kChains = 8;

// D-record update without folding: v_add_f32 + v_min_f32 per update (2 instructions).
__global__ __launch_bounds__(256) void valu_add_min(float *out, float c, int iters)
{
    float a[kChains], b[kChains];
    for (int j = 0; j < kChains; ++j) {
        a[j] = threadIdx.x * 0.5f + j;
        b[j] = 1e30f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < kChains; ++j) {
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(a[j]) : "v"(c));
            asm volatile("v_min_f32 %0, %0, %1" : "+v"(b[j]) : "v"(a[j]));
        }
    }
    float s = 0;
    for (int j = 0; j < kChains; ++j)
        s += b[j] + a[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// D-record update as built: two adds folded by one v_min3_f32 (3 instructions per 2 updates).
__global__ __launch_bounds__(256) void valu_add_add_min3(float *out, float c, int iters)
{
    float a[kChains], d[kChains], b[kChains];
    for (int j = 0; j < kChains; ++j) {
        a[j] = threadIdx.x * 0.5f + j;
        d[j] = threadIdx.x * 0.25f + j;
        b[j] = 1e30f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < kChains; ++j) {
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(a[j]) : "v"(c));
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(d[j]) : "v"(c));
            asm volatile("v_min3_f32 %0, %0, %1, %2" : "+v"(b[j]) : "v"(a[j]), "v"(d[j]));
        }
    }
    float s = 0;
    for (int j = 0; j < kChains; ++j)
        s += b[j] + a[j] + d[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Level-record update as built: add, compare, select of the level, min (4 instructions).
__global__ __launch_bounds__(256) void valu_add_cmp_sel_min(float *out, float c, int iters)
{
    float a[kChains], b[kChains];
    int g[kChains];
    for (int j = 0; j < kChains; ++j) {
        a[j] = threadIdx.x * 0.5f + j;
        b[j] = 1e30f;
        g[j] = 0;
    }
    for (int i = 0; i < iters; ++i) {
        int level = i;
        asm volatile("" : "+v"(level));
#pragma unroll
        for (int j = 0; j < kChains; ++j) {
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(a[j]) : "v"(c));
            asm volatile("v_cmp_lt_f32 vcc, %1, %2\n\tv_cndmask_b32 %0, %0, %3, vcc"
                         : "+v"(g[j])
                         : "v"(a[j]), "v"(b[j]), "v"(level)
                         : "vcc");
            asm volatile("v_min_f32 %0, %0, %1" : "+v"(b[j]) : "v"(a[j]));
        }
    }
    float s = 0;
    for (int j = 0; j < kChains; ++j)
        s += b[j] + a[j] + g[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Eight LDS reads of width sizeof(T) per iteration at immediate offsets; consecutive lanes read
// consecutive elements, the base moves by `step` dwords per iteration inside the buffer.
template <typename T>
__global__ __launch_bounds__(256) void lds_read(int *out, int step, int iters, int words)
{
    extern __shared__ __attribute__((aligned(16))) int lds[];
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
    CHECK(hipEventDestroy(a));
    CHECK(hipEventDestroy(b));
    return ms / reps;
}

int main()
{
    hipDeviceProp_t p;
    CHECK(hipGetDeviceProperties(&p, 0));
    const int cus = p.multiProcessorCount;
    const double clk = p.clockRate * 1e3;
    const int blocks = cus * 8, threads = 256;
    float *out;
    CHECK(hipMalloc(&out, sizeof(float) * blocks * threads));

    printf("{\"device\": \"%s\", \"compute_units\": %d, \"clock_mhz\": %.0f", p.gcnArchName, cus,
           clk / 1e6);
    auto valu = [&](const char *name, auto kernel, int instr_per_iter) {
        const float ms = time_ms(
            [&] { hipLaunchKernelGGL(kernel, dim3(blocks), dim3(threads), 0, 0, out, 1.0f, kIters); },
            20);
        const double ops = (double)blocks * threads * kIters * kChains * instr_per_iter;
        printf(", \"%s\": {\"ms\": %.4f, \"tlane_ops_per_s\": %.3f, \"lane_ops_per_clk_cu\": %.2f}",
               name, ms, ops / ms / 1e9, ops / (ms * 1e-3) / clk / cus);
    };
    valu("valu_add_min", valu_add_min, 2);
    valu("valu_add_add_min3", valu_add_add_min3, 3);
    valu("valu_add_cmp_sel_min", valu_add_cmp_sel_min, 4);

    const int words = 8192;    // 32 KB per workgroup, four workgroups (16 waves) per CU
    const int nb = cus * 4;
    auto lds = [&](const char *name, auto kernel, int width, int step) {
        CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, words * 4));
        const int iters = kIters / (width / 4);
        const float ms = time_ms(
            [&] {
                hipLaunchKernelGGL(kernel, dim3(nb), dim3(threads), words * 4, 0, (int *)out, step,
                                   iters, words);
            },
            10);
        const double bytes = (double)nb * threads * iters * 8 * width;
        printf(", \"%s\": {\"ms\": %.4f, \"tb_per_s\": %.2f, \"bytes_per_clk_cu\": %.1f}", name, ms,
               bytes / ms / 1e9, bytes / (ms * 1e-3) / clk / cus);
    };
    lds("lds_read_b32", lds_read<int>, 4, 65);
    lds("lds_read_b64", lds_read<int2>, 8, 66);
    lds("lds_read_b128", lds_read<int4>, 16, 68);
    printf("}\n");
    CHECK(hipFree(out));
    return 0;
}
