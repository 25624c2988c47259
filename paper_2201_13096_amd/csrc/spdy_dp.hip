// Batched dynamic program for the constrained layer-wise compression problem on gfx950.
//
// Sec. 3.2 (Eq. 2-3) and App. A (Alg. 1) define the computation; include/spdy_dp.h states the
// arithmetic contract (fp32, one add per update, smallest level / smallest t win ties).
//
// Mapping.  Alg. 1's triple loop (layer, level, time) is a min-plus recurrence with no reuse of a
// D_{l-1} element across levels (every level shifts the row by a different tau), so there is no
// contraction to put on the matrix cores: the work is one LDS read, one fp32 add, one compare
// and two selects per (l, s, t).  The remark after Alg. 1 (vectorise over t by shifting the row)
// is what the lanes do here:
//   * one workgroup owns one candidate; its two live D rows (previous / current layer) stay in
//     LDS for the whole solve and swap roles after every layer (one barrier per layer);
//   * the time axis is cut into chunks of 64 buckets; lane i of a wave works on bucket
//     64*c + i of a chunk, so every ds_read_b32 of the shifted row touches 64 consecutive
//     dwords (conflict-free for any shift) and every store of the level record is 64
//     consecutive bytes;
//   * a wave keeps R chunks in registers (running minimum and level for R buckets per lane) and
//     sweeps the levels once, with tau[l][s] and err[k][l][s] held in scalar registers;
//   * per (wave, level) the shift is classified with scalar compares: entirely left of the row
//     (skipped), entirely inside (no per-lane bounds test), or straddling t = tau (per-lane test).
// When two rows do not fit in LDS the same per-group routine runs from per-layer launches with
// the rows in global memory (they stay in L2 / Infinity Cache between consecutive layers).
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "spdy_dp.h"

namespace {

constexpr int kWave = 64;            // lanes per wavefront = buckets per chunk
constexpr int kMaxGroup = 10;        // most chunks a wave keeps in registers at once
constexpr int kResidentThreads = 1024;
constexpr int kStreamThreads = 256;  // per-layer kernel: 4 waves per workgroup
constexpr int kStreamGroup = 8;      // chunks per wave in the per-layer kernel
constexpr size_t kLdsBytes = 160 * 1024;
constexpr unsigned kNoLevel = 0xFF;
constexpr size_t kAlign = 256;

// ---------------------------------------------------------------------------------------------
// Workspace layout (host side, shared by every entry point)
struct Layout {
    int status;
    size_t row;          // buckets per padded row (multiple of 64)
    size_t choice_off;   // uint8 P[K][L][row]
    size_t tstar_off;    // int32 tstar[K]
    size_t drows_off;    // float D[2][K][row], only when !resident
    size_t total;
    bool resident;       // two D rows fit in LDS
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Layout make_layout(int K, int L, int S, int B)
{
    Layout lay{};
    if (K <= 0 || L <= 0 || S <= 0 || B < 0) {
        lay.status = SPDY_DP_ERR_DIM;
        return lay;
    }
    if (S > 255) {
        lay.status = SPDY_DP_ERR_LEVELS;
        return lay;
    }
    if (B > INT32_MAX - 2 * kWave * kMaxGroup) {   // bucket indices are int32 on the device
        lay.status = SPDY_DP_ERR_OVERFLOW;
        return lay;
    }
    lay.row = align_up((size_t)B + 1, kWave);
    // K * L * row and 2 * K * row * 4 must fit size_t with room to spare
    const unsigned __int128 cells = (unsigned __int128)K * (unsigned __int128)L * lay.row;
    const unsigned __int128 drows = (unsigned __int128)2 * K * lay.row * sizeof(float);
    if (cells + drows + (unsigned __int128)K * 4 + 4 * kAlign > (unsigned __int128)1 << 62) {
        lay.status = SPDY_DP_ERR_OVERFLOW;
        return lay;
    }
    lay.resident = 2 * lay.row * sizeof(float) <= kLdsBytes;
    lay.choice_off = 0;
    lay.tstar_off = align_up((size_t)cells, kAlign);
    lay.drows_off = align_up(lay.tstar_off + (size_t)K * sizeof(int32_t), kAlign);
    lay.total = lay.resident ? lay.drows_off : lay.drows_off + (size_t)drows;
    lay.status = SPDY_DP_OK;
    return lay;
}

// ---------------------------------------------------------------------------------------------
// One group of R chunks (R*64 consecutive buckets starting at t0) of one layer.
// prev / cur: the two D rows (LDS or global); choice: this layer's row of the level record.
// tau_l / err_l: the S times and errors of this layer for this candidate (wave-uniform).
template <int R>
__device__ __forceinline__ void fill_group(const float *__restrict__ prev, float *__restrict__ cur,
                                           uint8_t *__restrict__ choice,
                                           const int32_t *__restrict__ tau_l,
                                           const float *__restrict__ err_l, int S, int t0,
                                           int lane)
{
    float best[R];
    unsigned arg[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        best[j] = __builtin_inff();
        arg[j] = kNoLevel;
    }
    const int tl = t0 + lane;                 // this lane's bucket in chunk 0 of the group
    const int last = t0 + R * kWave - 1;      // last bucket of the group

    for (int s = 0; s < S; ++s) {
        const int ts = tau_l[s];
        const float es = err_l[s];
        if (ts > last)
            continue;                         // every lane would read left of t = 0
        if (ts <= t0) {                       // every lane reads inside the row
            const float *p = prev + (tl - ts);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const float v = p[j * kWave] + es;
                if (v < best[j]) {
                    best[j] = v;
                    arg[j] = (unsigned)s;
                }
            }
        } else {                              // the group straddles t = tau: test per lane
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int u = tl + j * kWave - ts;
                if (u >= 0) {
                    const float v = prev[u] + es;
                    if (v < best[j]) {
                        best[j] = v;
                        arg[j] = (unsigned)s;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
        cur[tl + j * kWave] = best[j];
        choice[tl + j * kWave] = (uint8_t)arg[j];
    }
}

// Chunks [c, c_end) of one layer, in groups of at most kMaxGroup chunks of near-equal size.
__device__ __forceinline__ void fill_chunks(const float *prev, float *cur, uint8_t *choice,
                                            const int32_t *tau_l, const float *err_l, int S,
                                            int c, int c_end, int lane)
{
    while (c < c_end) {
        const int n = c_end - c;
        const int groups = (n + kMaxGroup - 1) / kMaxGroup;
        const int r = (n + groups - 1) / groups;
        const int t0 = c * kWave;
        switch (r) {
#define SPDY_CASE(RR)                                                                 \
    case RR:                                                                          \
        fill_group<RR>(prev, cur, choice, tau_l, err_l, S, t0, lane);                 \
        break;
            SPDY_CASE(1)
            SPDY_CASE(2)
            SPDY_CASE(3)
            SPDY_CASE(4)
            SPDY_CASE(5)
            SPDY_CASE(6)
            SPDY_CASE(7)
            SPDY_CASE(8)
            SPDY_CASE(9)
            SPDY_CASE(10)
#undef SPDY_CASE
        }
        c += r;
    }
}

// (value, t) pairs ordered by value, then by smaller t.
__device__ __forceinline__ void argmin_merge(float &bv, int &bt, float v, int t)
{
    if (v < bv || (v == bv && t < bt)) {
        bv = v;
        bt = t;
    }
}

// Smallest t <= B attaining min_t row[t], reduced over the workgroup.  scratch_v / scratch_t: one
// word per wave each, in LDS, not aliasing row.  Result valid in thread 0.
__device__ __forceinline__ void block_argmin(const float *row, int B, float *scratch_v,
                                             int *scratch_t, float &out_v, int &out_t)
{
    const int tid = threadIdx.x, nthreads = blockDim.x;
    float bv = __builtin_inff();
    int bt = INT32_MAX;
    for (int t = tid; t <= B; t += nthreads)
        argmin_merge(bv, bt, row[t], t);
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float ov = __shfl_down(bv, off, kWave);
        const int ot = __shfl_down(bt, off, kWave);
        argmin_merge(bv, bt, ov, ot);
    }
    const int wave = tid / kWave, nwaves = nthreads / kWave;
    if ((tid & (kWave - 1)) == 0) {
        scratch_v[wave] = bv;
        scratch_t[wave] = bt;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < nwaves; ++w)
            argmin_merge(bv, bt, scratch_v[w], scratch_t[w]);
        out_v = bv;
        out_t = bt;
    }
}

// ---------------------------------------------------------------------------------------------
// Resident path: one workgroup per candidate, both D rows in LDS for all L layers.
__global__ __launch_bounds__(kResidentThreads, 8) void dp_fill_resident(
    const int32_t *__restrict__ tau, const float *__restrict__ err, int L, int S, int B, int row,
    uint8_t *__restrict__ choice, int32_t *__restrict__ tstar, float *__restrict__ cost)
{
    extern __shared__ float lds[];
    float *row0 = lds;
    float *row1 = lds + row;

    const int k = blockIdx.x;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nwaves = nthreads / kWave;

    // D before the first layer: time 0 costs nothing, nothing else is reachable (Eq. 3 then is
    // the general update).  -0.0f + e returns e bit for bit for every e, +0.0f would not for
    // e = -0.0f.
    for (int t = tid; t < row; t += nthreads)
        row0[t] = (t == 0) ? -0.0f : __builtin_inff();
    __syncthreads();

    const int nchunks = row / kWave;
    const int c_begin = (int)((long long)wave * nchunks / nwaves);
    const int c_end = (int)((long long)(wave + 1) * nchunks / nwaves);
    const float *err_k = err + (size_t)k * L * S;
    uint8_t *choice_k = choice + (size_t)k * L * row;

    for (int l = 0; l < L; ++l) {
        const float *prev = (l & 1) ? row1 : row0;
        float *cur = (l & 1) ? row0 : row1;
        fill_chunks(prev, cur, choice_k + (size_t)l * row, tau + (size_t)l * S,
                    err_k + (size_t)l * S, S, c_begin, c_end, lane);
        __syncthreads();
    }

    const float *last = (L & 1) ? row1 : row0;
    float *scratch = (L & 1) ? row0 : row1;   // the other row is dead now
    float bv;
    int bt;
    block_argmin(last, B, scratch, reinterpret_cast<int *>(scratch) + kResidentThreads / kWave, bv, bt);
    if (tid == 0) {
        cost[k] = bv;
        tstar[k] = (bv < __builtin_inff()) ? bt : -1;   // -1: no profile meets the budget
    }
}

// ---------------------------------------------------------------------------------------------
// Streamed path (two rows exceed LDS): D rows live in global memory, one launch per layer.
__global__ void dp_init_rows(float *__restrict__ d0, int row, int K)
{
    const size_t n = (size_t)K * row;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        d0[i] = (i % row == 0) ? -0.0f : __builtin_inff();
}

__global__ __launch_bounds__(kStreamThreads) void dp_layer_streamed(
    const int32_t *__restrict__ tau_l, const float *__restrict__ err_l0, int L, int S, int row,
    const float *__restrict__ dprev, float *__restrict__ dcur, uint8_t *__restrict__ choice_l0)
{
    const int k = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int nchunks = row / kWave;
    const int c = (blockIdx.y * (kStreamThreads / kWave) + wave) * kStreamGroup;
    if (c >= nchunks)
        return;
    const int c_end = min(c + kStreamGroup, nchunks);
    fill_chunks(dprev + (size_t)k * row, dcur + (size_t)k * row,
                choice_l0 + (size_t)k * L * row, tau_l, err_l0 + (size_t)k * L * S, S, c, c_end,
                lane);
}

__global__ __launch_bounds__(kStreamThreads) void dp_final_argmin(
    const float *__restrict__ dlast, int row, int B, int32_t *__restrict__ tstar,
    float *__restrict__ cost)
{
    __shared__ float sv[kStreamThreads / kWave];
    __shared__ int st[kStreamThreads / kWave];
    const int k = blockIdx.x;
    float bv;
    int bt;
    block_argmin(dlast + (size_t)k * row, B, sv, st, bv, bt);
    if (threadIdx.x == 0) {
        cost[k] = bv;
        tstar[k] = (bv < __builtin_inff()) ? bt : -1;   // -1: no profile meets the budget
    }
}

// ---------------------------------------------------------------------------------------------
// Walk back (last loop of Alg. 1): one lane per candidate, L dependent one-byte reads.
__global__ void dp_backtrace(const int32_t *__restrict__ tau, const uint8_t *__restrict__ choice,
                             const int32_t *__restrict__ tstar, int K, int L, int S, int row, int16_t *__restrict__ profile)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K)
        return;
    int16_t *prof = profile + (size_t)k * L;
    int t = tstar[k];
    if (t < 0) {
        for (int l = 0; l < L; ++l)
            prof[l] = -1;
        return;
    }
    const uint8_t *choice_k = choice + (size_t)k * L * row;
    for (int l = L - 1; l >= 0; --l) {
        const int s = choice_k[(size_t)l * row + t];
        prof[l] = (int16_t)s;
        if (s >= S)          // cannot happen on a filled table; never index tau out of range
            break;
        t -= tau[(size_t)l * S + s];
        if (t < 0)
            break;
    }
}

int check_common(const Layout &lay, const void *workspace, size_t workspace_bytes)
{
    if (lay.status != SPDY_DP_OK)
        return lay.status;
    if (!workspace)
        return SPDY_DP_ERR_NULL;
    if (workspace_bytes < lay.total)
        return SPDY_DP_ERR_WORKSPACE;
    return SPDY_DP_OK;
}

int launch_status()
{
    return hipGetLastError() == hipSuccess ? SPDY_DP_OK : SPDY_DP_ERR_LAUNCH;
}

}  // namespace

extern "C" {

size_t spdy_dp_workspace_bytes(int K, int L, int S, int B)
{
    const Layout lay = make_layout(K, L, S, B);
    return lay.status == SPDY_DP_OK ? lay.total : 0;
}

int spdy_dp_workspace_layout(int K, int L, int S, int B, size_t *choice_offset,
                             size_t *choice_pitch, size_t *tstar_offset)
{
    if (!choice_offset || !choice_pitch || !tstar_offset)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B);
    if (lay.status != SPDY_DP_OK)
        return lay.status;
    *choice_offset = lay.choice_off;
    *choice_pitch = lay.row;
    *tstar_offset = lay.tstar_off;
    return SPDY_DP_OK;
}

int spdy_dp_fill(const int32_t *tau, const float *err, int K, int L, int S, int B, float *cost,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!tau || !err || !cost)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B);
    const int st = check_common(lay, workspace, workspace_bytes);
    if (st != SPDY_DP_OK)
        return st;
    hipStream_t q = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    uint8_t *choice = reinterpret_cast<uint8_t *>(ws + lay.choice_off);
    int32_t *tstar = reinterpret_cast<int32_t *>(ws + lay.tstar_off);
    const int row = (int)lay.row;
    const int nchunks = row / kWave;
    (void)hipGetLastError();

    if (lay.resident) {
        const size_t lds = 2 * lay.row * sizeof(float);
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(dp_fill_resident),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return SPDY_DP_ERR_LAUNCH;
        const int waves = nchunks < kResidentThreads / kWave ? nchunks : kResidentThreads / kWave;
        hipLaunchKernelGGL(dp_fill_resident, dim3(K), dim3(waves * kWave), lds, q, tau, err, L, S,
                           B, row, choice, tstar, cost);
        return launch_status();
    }

    float *d0 = reinterpret_cast<float *>(ws + lay.drows_off);
    float *d1 = d0 + (size_t)K * lay.row;
    hipLaunchKernelGGL(dp_init_rows, dim3(1024), dim3(256), 0, q, d0, row, K);
    const int chunks_per_block = (kStreamThreads / kWave) * kStreamGroup;
    const dim3 grid(K, (nchunks + chunks_per_block - 1) / chunks_per_block);
    for (int l = 0; l < L; ++l) {
        const float *prev = (l & 1) ? d1 : d0;
        float *cur = (l & 1) ? d0 : d1;
        hipLaunchKernelGGL(dp_layer_streamed, grid, dim3(kStreamThreads), 0, q,
                           tau + (size_t)l * S, err + (size_t)l * S, L, S, row, prev, cur,
                           choice + (size_t)l * lay.row);
    }
    hipLaunchKernelGGL(dp_final_argmin, dim3(K), dim3(kStreamThreads), 0, q,
                       (L & 1) ? d1 : d0, row, B, tstar, cost);
    return launch_status();
}

int spdy_dp_backtrace(const int32_t *tau, int K, int L, int S, int B, int16_t *profile,
                      const void *workspace, size_t workspace_bytes, void *stream)
{
    if (!tau || !profile)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B);
    const int st = check_common(lay, workspace, workspace_bytes);
    if (st != SPDY_DP_OK)
        return st;
    hipStream_t q = static_cast<hipStream_t>(stream);
    const char *ws = static_cast<const char *>(workspace);
    const uint8_t *choice = reinterpret_cast<const uint8_t *>(ws + lay.choice_off);
    const int32_t *tstar = reinterpret_cast<const int32_t *>(ws + lay.tstar_off);
    (void)hipGetLastError();
    hipLaunchKernelGGL(dp_backtrace, dim3((K + kWave - 1) / kWave), dim3(kWave), 0, q, tau,
                       choice, tstar, K, L, S, (int)lay.row, profile);
    return launch_status();
}

int spdy_dp_solve_batched(const int32_t *tau, const float *err, int K, int L, int S, int B,
                          int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!tau || !err || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    int st = spdy_dp_fill(tau, err, K, L, S, B, cost, workspace, workspace_bytes, stream);
    if (st != SPDY_DP_OK)
        return st;
    return spdy_dp_backtrace(tau, K, L, S, B, profile, workspace, workspace_bytes, stream);
}

const char *spdy_dp_strerror(int status)
{
    switch (status) {
    case SPDY_DP_OK: return "ok";
    case SPDY_DP_ERR_NULL: return "a required pointer is NULL";
    case SPDY_DP_ERR_DIM: return "K, L and S must be positive and B non-negative";
    case SPDY_DP_ERR_LEVELS: return "S exceeds 255 levels (one byte per recorded level)";
    case SPDY_DP_ERR_WORKSPACE: return "workspace smaller than spdy_dp_workspace_bytes()";
    case SPDY_DP_ERR_OVERFLOW: return "problem size overflows the index arithmetic";
    case SPDY_DP_ERR_LAUNCH: return "HIP runtime refused a kernel launch";
    default: return "unknown status";
    }
}

}  // extern "C"
