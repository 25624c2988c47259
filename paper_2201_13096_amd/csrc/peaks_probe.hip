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

// The sweep of the fill kernel by itself (no barriers, no record stores, no table hand-over): a
// wave keeps a running minimum per bucket and visits pairs of entries; per pair and bucket one
// LDS read and one add per entry and one v_min3.  Two layouts:
//   sweep_b32:  lane = bucket, 16 chunks of 64 buckets per wave, 32-bit reads;
//   sweep_b128: lane = four consecutive buckets, 4 chunks of 256 buckets per wave, one aligned
//               128-bit read per entry; a shift that is not a multiple of four takes its last
//               kRes values from the lane to the left with the add (DPP wave_shr:1).
// Eight waves per workgroup, two workgroups per compute unit, as the fill runs.
constexpr int kSweepRow = 8 * 16 * 64;   // floats swept per workgroup
constexpr int kSweepHalo = 2048;         // shifts stay below this
typedef float float4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void min3(float &b, float x, float y)
{
    asm("v_min3_f32 %0, %0, %1, %2" : "+v"(b) : "v"(x), "v"(y));
}
__device__ __forceinline__ float from_left(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_float(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__global__ __launch_bounds__(512, 2) void sweep_b32(float *out, const int *shifts,
                                                    const float *errs, int pairs, int iters)
{
    extern __shared__ __attribute__((aligned(16))) float row[];
    for (int i = threadIdx.x; i < kSweepRow + kSweepHalo; i += blockDim.x)
        row[i] = (float)(i & 1023);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *mine = row + kSweepHalo + wave * 16 * 64 + lane;
    float best[16];
    for (int j = 0; j < 16; ++j)
        best[j] = 1e30f;
    const int sh = shifts[lane];
    const float er = errs[lane];
    for (int it = 0; it < iters; ++it)
        for (int i = 0; i < 2 * pairs; i += 2) {
            const float *p0 = mine - __builtin_amdgcn_readlane(sh, i);
            const float *p1 = mine - __builtin_amdgcn_readlane(sh, i + 1);
            const float e0 = lane_float(er, i), e1 = lane_float(er, i + 1);
#pragma unroll
            for (int j = 0; j < 16; ++j)
                min3(best[j], p0[j * 64] + e0, p1[j * 64] + e1);
        }
    float s = 0;
    for (int j = 0; j < 16; ++j)
        s += best[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int kRes>
__global__ __launch_bounds__(512, 2) void sweep_b128(float *out, const int *shifts,
                                                     const float *errs, int pairs, int iters)
{
    extern __shared__ __attribute__((aligned(16))) float row[];
    for (int i = threadIdx.x; i < kSweepRow + kSweepHalo; i += blockDim.x)
        row[i] = (float)(i & 1023);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float4v *mine = reinterpret_cast<const float4v *>(row + kSweepHalo) + wave * 4 * 64 + lane;
    float best[4][4];
    for (int j = 0; j < 4; ++j)
        for (int c = 0; c < 4; ++c)
            best[j][c] = 1e30f;
    const int sh = shifts[lane] >> 2;    // in quads
    const float er = errs[lane];
    for (int it = 0; it < iters; ++it)
        for (int i = 0; i < 2 * pairs; i += 2) {
            const float4v *p0 = mine - __builtin_amdgcn_readlane(sh, i);
            const float4v *p1 = mine - __builtin_amdgcn_readlane(sh, i + 1);
            float e0 = lane_float(er, i), e1 = lane_float(er, i + 1);
            asm volatile("" : "+v"(e0), "+v"(e1));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4v a = p0[j * 64], b = p1[j * 64];
                const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float x = (c >= kRes ? av[c - kRes] : from_left(av[4 + c - kRes])) + e0;
                    const float y = (c >= kRes ? bv[c - kRes] : from_left(bv[4 + c - kRes])) + e1;
                    min3(best[j][c], x, y);
                }
            }
        }
    float s = 0;
    for (int j = 0; j < 4; ++j)
        for (int c = 0; c < 4; ++c)
            s += best[j][c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
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
    {
        // the bare sweep: updates per clock per compute unit
        const int pairs = 16, iters = 64, wgs = cus * 2, wg_threads = 512;
        int hs[64];
        float he[64];
        for (int i = 0; i < 64; ++i) {
            hs[i] = (i * 52 + 7) & ~3;
            if (hs[i] > kSweepHalo - 64)
                hs[i] = kSweepHalo - 64;
            he[i] = 0.25f * i;
        }
        int *sh;
        float *er;
        CHECK(hipMalloc(&sh, sizeof hs));
        CHECK(hipMalloc(&er, sizeof he));
        CHECK(hipMemcpy(sh, hs, sizeof hs, hipMemcpyHostToDevice));
        CHECK(hipMemcpy(er, he, sizeof he, hipMemcpyHostToDevice));
        const size_t bytes = (kSweepRow + kSweepHalo) * sizeof(float);
        const double updates = (double)wgs * wg_threads * 16 * (2.0 * pairs) * iters;
        auto sweep = [&](auto kernel) {
            CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
            const float ms = time_ms(
                [&] {
                    hipLaunchKernelGGL(kernel, dim3(wgs), dim3(wg_threads), bytes, 0, out, sh, er,
                                       pairs, iters);
                },
                20);
            return updates / (ms * 1e-3) / clk / cus;
        };
        const double u32 = sweep(sweep_b32);
        const double u0 = sweep(sweep_b128<0>), u1 = sweep(sweep_b128<1>);
        const double u2 = sweep(sweep_b128<2>), u3 = sweep(sweep_b128<3>);
        printf(", \"sweep_b32\": {\"updates_per_clk_cu\": %.2f}", u32);
        printf(", \"sweep_b128\": {\"updates_per_clk_cu\": %.2f, \"by_shift_mod_4\": [%.2f, %.2f, %.2f, "
               "%.2f]}",
               4.0 / (1.0 / u0 + 1.0 / u1 + 1.0 / u2 + 1.0 / u3), u0, u1, u2, u3);
        CHECK(hipFree(sh));
        CHECK(hipFree(er));
    }
    printf("}\n");
    CHECK(hipFree(out));
    return 0;
}
