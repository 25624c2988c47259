/*
 * spdy_dp -- batched solver for the constrained layer-wise compression problem on one AMD
 * MI355X (gfx950) GPU.
 *
 * Problem (Sec. 3.1, Eq. 1).  A model has L layers; layer l can be compressed to one of S levels;
 * level s of layer l costs an integer time tau[l][s] (Sec. 3.2: time discretised into B buckets,
 * so the budget is T = B) and an error err[k][l][s].  For every candidate error table k the
 * solver returns levels s_0..s_{L-1} minimising  sum_l err[k][l][s_l]  subject to
 * sum_l tau[l][s_l] <= B.  All K candidates share the one timing table (they are the error
 * tables a coefficient search proposes for one model, Sec. 3.3).
 *
 * Method (Sec. 3.2, Eq. 2-3; App. A, Alg. 1).  Bottom-up dynamic programming over time:
 *     D_l[t] = min_s ( D_{l-1}[t - tau[l][s]] + err[k][l][s] ),   t = 0..B,
 * where D_l[t] is the least error of layers 0..l taking exactly time t, the first layer places
 * err[k][0][s] at t = tau[0][s], the level attaining the minimum is recorded per cell, the
 * answer is min_{t<=B} D_{L-1}[t], and the recorded levels are walked back from that cell.
 *
 * Arithmetic contract (fixes what the text leaves open so results are reproducible bit for bit):
 *   - D is fp32; each update is ONE round-to-nearest fp32 add; layers are accumulated in order
 *     0..L-1, so cost[k] equals the left-to-right fp32 sum of err over the returned profile;
 *     subnormals are kept;
 *   - within a cell the smallest level index among equal values wins (strict "<" in Alg. 1 with
 *     levels visited in ascending order);
 *   - the final argmin over t returns the smallest t among equal values;
 *   - a level with tau > B, or with err = +inf, is never chosen; tau = 0 is legal;
 *   - a candidate that no profile satisfies gets cost = +inf and profile = -1 (status stays OK).
 *
 * Exact reductions of Alg. 1's table are applied on the device (results are unchanged):
 *   - every layer's smallest time m_l = min_s tau[l][s] is subtracted from that layer's times
 *     and M = sum_l m_l from the budget, so layer l's row only spans t' = t - (m_0 + .. + m_l)
 *     in [0, B - M] (cells outside can never lie on a profile that meets the budget);
 *   - cells beyond the largest time reachable after l layers are +inf and are not computed;
 *   - levels of a layer that take the same time read the same cell of D_{l-1}, and a rounded
 *     add is monotone in the addend: when D itself is recorded they are served by one update
 *     with the smallest of their errors (the walk back still picks the smallest level); when
 *     the level is recorded, a level is not visited if an earlier one of the same time has an
 *     error no larger (the strict "<" could never select it).
 *
 * What is recorded per cell for the walk back depends on the workspace the caller provides:
 *   - spdy_dp_workspace_bytes():     D itself (fp32 per cell); the fill then needs only an add
 *     and a min per update, and the walk back re-derives the level of the L cells on the path
 *     (smallest s with D_{l-1}[t - tau[l][s]] + err[k][l][s] == D_l[t]);
 *   - spdy_dp_workspace_bytes_min(): the level P of Alg. 1 (one byte per cell, 4x smaller; the
 *     fill tracks the level with a compare and two selects per update).
 * Both give the same profile and cost, bit for bit.
 *
 * Conventions for every entry point:
 *   - tau, err, profile, cost, workspace are DEVICE pointers, C-contiguous, owned by the caller.
 *     The library allocates nothing, frees nothing and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and results are valid
 *     once the caller has synchronised that stream.  Calls on different streams must not share a
 *     workspace.
 *   - Arguments are validated on the host; on a negative return other than SPDY_DP_ERR_LAUNCH
 *     nothing was enqueued and no output was touched.  The CONTENTS of tau and err are not
 *     inspected (that would need a device-to-host copy): tau[l][s] < 0, err = NaN and err = -inf
 *     are undefined behaviour.
 *   - The device in use must be a gfx950; the current HIP device is used.
 */
#ifndef SPDY_DP_H
#define SPDY_DP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPDY_DP_OK 0
#define SPDY_DP_ERR_NULL (-1)      /* a required pointer is NULL                              */
#define SPDY_DP_ERR_DIM (-2)       /* K, L or S <= 0, or B < 0                                 */
#define SPDY_DP_ERR_LEVELS (-3)    /* S > 255: a recorded level is one byte, 0xFF = "no level
                                      reaches this cell"                                        */
#define SPDY_DP_ERR_WORKSPACE (-4) /* workspace_bytes < spdy_dp_workspace_bytes_min(K,L,S,B)   */
#define SPDY_DP_ERR_OVERFLOW (-5)  /* K * L * (B + 1) does not fit the index arithmetic         */
#define SPDY_DP_ERR_LAUNCH (-9)    /* the HIP runtime refused a query or a launch (see
                                      hipGetLastError); unlike the argument errors above it can
                                      come back after earlier kernels of the call were enqueued,
                                      so the outputs are then undefined                          */
#define SPDY_DP_ERR_STATIC_LIMIT (-10) /* spdy_dp_solve_batched_static: the problem needs more
                                      than SPDY_DP_STATIC_WORKSPACE_BYTES of workspace           */

/* Size of the workspace built into the library for spdy_dp_solve_batched_static (64 MiB of
 * device memory per GPU the library runs on, held until the process ends). */
#define SPDY_DP_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)

/* Bytes of device workspace for the fast variant (fp32 D recorded per cell), or 0 if the sizes
 * are invalid.  About 4 * K * L * (B + 1) bytes, plus 8 * K * (B + 1) when two rows of B + 1 floats
 * exceed the 160 KB of LDS of a compute unit. */
size_t spdy_dp_workspace_bytes(int K, int L, int S, int B);

/* Smallest workspace accepted (one-byte level record per cell), or 0 if the sizes are invalid.
 * About K * L * (B + 1) bytes, plus the same 8 * K * (B + 1) for long rows.  Any size in between
 * selects this variant too. */
size_t spdy_dp_workspace_bytes_min(int K, int L, int S, int B);

/* Solve all K candidates: the whole of Alg. 1 (table fill, final argmin over t, walk back).
 *   tau      in  int32 [L][S]     times in buckets, >= 0, shared by all candidates
 *   err      in  fp32  [K][L][S]  errors, finite or +inf
 *   profile  out int16 [K][L]     chosen level per layer in [0, S), or -1 if infeasible
 *   cost     out fp32  [K]        optimal error, +inf if infeasible
 * Equivalent to spdy_dp_fill followed by spdy_dp_backtrace on the same stream. */
int spdy_dp_solve_batched(const int32_t *tau, const float *err, int K, int L, int S, int B,
                          int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                          void *stream);

/* spdy_dp_solve_batched for callers that cannot allocate device memory or be handed a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is a fixed array of SPDY_DP_STATIC_WORKSPACE_BYTES inside the library's code object
 * (one copy per GPU); this call allocates nothing, frees nothing and calls no allocating routine.
 * Arguments, outputs and results are those of spdy_dp_solve_batched; the D record is used when
 * spdy_dp_workspace_bytes(K, L, S, B) fits the array, the level record when only
 * spdy_dp_workspace_bytes_min does, and SPDY_DP_ERR_STATIC_LIMIT is returned (nothing enqueued)
 * when neither does (one ResNet-50-sized table, L = 54, S = 40, B = 10^4, takes 2.2 MB with the
 * D record: 30 such candidates fit, 123 with the level record).
 * Every call on a GPU uses that GPU's one array, whatever the stream: calls that overlap in time
 * on one GPU race and return garbage; order them on one stream or with events.  Nothing needs
 * clearing between calls (no kernel assumes anything about the array's contents). */
int spdy_dp_solve_batched_static(const int32_t *tau, const float *err, int K, int L, int S, int B,
                                 int16_t *profile, float *cost, void *stream);

/* First part of Alg. 1: fills the tables layer by layer (Eq. 2-3), records D or the chosen level
 * of every computed cell in the workspace, and takes the final argmin over t <= B.  Writes
 * cost[k] (compares equal to the final cost; spdy_dp_backtrace rewrites it) and keeps t*[k] in
 * the workspace. */
int spdy_dp_fill(const int32_t *tau, const float *err, int K, int L, int S, int B, float *cost,
                 void *workspace, size_t workspace_bytes, void *stream);

/* Last loop of Alg. 1: walks back from (L-1, t*[k]) and writes profile[k] and cost[k].
 * `workspace` (same size) must be the one a spdy_dp_fill call with the same tau, err, K, L, S, B
 * has filled earlier on the same stream (or on a stream already synchronised with it). */
int spdy_dp_backtrace(const int32_t *tau, const float *err, int K, int L, int S, int B,
                      int16_t *profile, float *cost, const void *workspace,
                      size_t workspace_bytes, void *stream);

/* spdy_dp_solve_batched for error tables of the form of Eq. 4: err[k][l][s] = c[k][l] * w[s],
 * a per-layer sensitivity times a fixed per-level weight (Eq. 4: w_i = (i / (S - 1))^2).  The
 * product is formed on the device with one round-to-nearest fp32 multiply wherever an error is
 * needed, so the K * L * S table never exists in memory; results equal spdy_dp_solve_batched on
 * the table err = fl32(c * w), bit for bit.
 *   c  in  fp32 [K][L]  sensitivities, finite (inf * 0 would be NaN)
 *   w  in  fp32 [S]     level weights, finite
 * Workspace, outputs and status codes as for spdy_dp_solve_batched. */
int spdy_dp_solve_sensitivities(const int32_t *tau, const float *c, const float *w, int K, int L,
                                int S, int B, int16_t *profile, float *cost, void *workspace,
                                size_t workspace_bytes, void *stream);

/* Several budgets from one fill.  D_l[t] is the least error at EXACTLY time t (Eq. 2-3), so the
 * table does not depend on the budget: it is filled once for max_j budgets[j], and for every
 * budget the final argmin runs over t <= budgets[j] and the levels are walked back from there
 * (profiles for a range of speed-up targets at the cost of one fill).  Results equal J separate
 * spdy_dp_solve_batched calls, bit for bit.
 *   budgets  in  int32 [J]        HOST pointer, each >= 0
 *   profile  out int16 [J][K][L]  device
 *   cost     out fp32  [J][K]     device
 * The workspace must have at least spdy_dp_workspace_bytes(K, L, S, max budget) bytes (the D
 * record keeps the last row the argmin needs); a smaller one returns SPDY_DP_ERR_WORKSPACE. */
int spdy_dp_solve_budgets(const int32_t *tau, const float *err, int K, int L, int S,
                          const int32_t *budgets, int J, int16_t *profile, float *cost,
                          void *workspace, size_t workspace_bytes, void *stream);

/* Re-solve K candidates that share their first layers with an already solved incumbent.  The
 * coefficient search (Sec. 3.3, Alg. 4) proposes candidates by resampling a few sensitivities of
 * the incumbent, so candidate k's errors equal the incumbent's for every layer before the first
 * resampled one; D_l depends on layers 0..l only (Eq. 2), so those rows are the incumbent's and
 * the fill starts at layer first_layer[k] from the incumbent's recorded row.  Results equal
 * spdy_dp_solve_batched on the same err, bit for bit.
 *   err          in  fp32 [K][L][S]  full tables; the CALLER guarantees err[k][l][:] equals the
 *                                   incumbent's err[l][:] bit for bit for l < first_layer[k]
 *   first_layer  in  int32 [K]       DEVICE; values are clamped to [0, L] (0 = solve from scratch,
 *                                   L = identical to the incumbent)
 *   incumbent_workspace              DEVICE; the workspace of a finished spdy_dp_solve_batched /
 *                                   spdy_dp_fill call with K = 1, the same tau, L, S, B, and at
 *                                   least spdy_dp_workspace_bytes(1, L, S, B) bytes (D record);
 *                                   it is only read
 * `workspace` (distinct from the incumbent's) needs spdy_dp_workspace_bytes(K, L, S, B) bytes; a
 * smaller one of either returns SPDY_DP_ERR_WORKSPACE.  Candidates of one workgroup step through
 * the layers together, so sorting the candidates by first_layer wastes the least. */
int spdy_dp_solve_from_incumbent(const int32_t *tau, const float *err, const int32_t *first_layer,
                                 int K, int L, int S, int B, const void *incumbent_workspace,
                                 size_t incumbent_bytes, int16_t *profile, float *cost,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* The same solve with a fraction of the record.  Sec. 3.2 gives the dynamic program O(L T)
 * memory for its matrices; this variant keeps about 2 sqrt(L) rows of D per candidate instead
 * of L and pays with a second fill: a first pass over all layers keeps every stride-th row
 * (checkpoints) and finds the final time, then each block of `stride` layers, the last one
 * first, is filled again from the checkpoint below it and walked back.  Results equal
 * spdy_dp_solve_batched bit for bit.
 *   stride   layers per block; <= 0 picks ceil(sqrt(L)); values above L act as L
 * Workspace: spdy_dp_workspace_bytes_checkpointed(K, L, S, B, stride) bytes with the SAME stride
 * (about 4 * K * (L / stride + stride) * (B + 1)); a smaller one returns SPDY_DP_ERR_WORKSPACE.
 * Everything else is as for spdy_dp_solve_batched. */
size_t spdy_dp_workspace_bytes_checkpointed(int K, int L, int S, int B, int stride);
int spdy_dp_solve_checkpointed(const int32_t *tau, const float *err, int K, int L, int S, int B,
                               int stride, int16_t *profile, float *cost, void *workspace,
                               size_t workspace_bytes, void *stream);

/* Test/debug accessor: where things are in a workspace of `workspace_bytes` bytes.
 *   out[0] variant: 0 = fp32 D record, 1 = one-byte level record
 *   out[1] byte offset of the int32 header: [0] B - M (or -1 if M > B: nobody is feasible),
 *          [1] M, [2] reduced row length (B - M + 1 padded to 64), [3] which launch of the fill
 *          did the work: 0 rows in global memory, 1 one row per candidate in LDS updated in
 *          place, 2 two rows in LDS, 3 / 4 as 1 / 0 in a workgroup of twice the waves (D record:
 *          rows too long for launch 1); [4] waves per candidate, [5] candidates per workgroup,
 *          [6] 1 if rows are updated in place; and what that choice was made from: [7] bytes of
 *          LDS for the windows of launch 0, [8] waves per workgroup, [9] most 64-bucket chunks a
 *          wave keeps in registers, [10] / [11] dynamic LDS bytes of launches 1 / 2 (0: not
 *          enqueued), [12] floats of +inf apron left of a row, [13] 1 if launch 1 ran with
 *          twice the waves of [8], the second half dividing each layer's levels with the first
 *          (D record, S <= 64, no more candidates than compute units), [14] waves of launch 3
 *          (0: not enqueued), [15] most chunks one of them keeps in registers, [16] its dynamic
 *          LDS bytes, [17] waves of the global-row launch.  Per-layer arrays follow the
 *          out[6] header words: m_l at [out[6] + l], the number of computed 64-bucket chunks of
 *          layer l at [out[6] + L + l], the largest usable shift of layer l at
 *          [out[6] + (2 + out[7]) L + l]
 *   out[2] byte offset of int32 t*[K] (reduced time t* - M, or -1 if infeasible)
 *   out[3] byte offset of the record
 *   out[4] record pitch in elements (buckets per row, a multiple of 64)
 *   out[5] record rows per candidate (L: row l holds layer l)
 *   out[6] int32 words of the header before its per-layer arrays
 *   out[7] int32 words per layer of the wave plan that sits between the second and the last
 *          per-layer array
 * Element (k, l, t') of the record is at out[3] + ((k * out[5] + l) * out[4] + t') * elemsize.
 * Returns SPDY_DP_OK or a size / workspace error. */
int spdy_dp_workspace_layout(int K, int L, int S, int B, size_t workspace_bytes, size_t out[8]);

/* Static, human-readable text for a status code. */
const char *spdy_dp_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPDY_DP_H */
