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
 * Conventions for every entry point:
 *   - tau, err, profile, cost, workspace are DEVICE pointers, C-contiguous, owned by the caller.
 *     The library allocates nothing, frees nothing and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and results are valid
 *     once the caller has synchronised that stream.  Calls on different streams must not share a
 *     workspace.
 *   - Arguments are validated on the host; on a negative return nothing was enqueued and no
 *     output was touched.  The CONTENTS of tau and err are not inspected (that would need a
 *     device-to-host copy): tau[l][s] < 0, err = NaN and err = -inf are undefined behaviour.
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
#define SPDY_DP_ERR_LEVELS (-3)    /* S > 255: the per-cell level record is one byte, 0xFF =
                                      "no level reaches this cell"                              */
#define SPDY_DP_ERR_WORKSPACE (-4) /* workspace_bytes < spdy_dp_workspace_bytes(K, L, S, B)    */
#define SPDY_DP_ERR_OVERFLOW (-5)  /* K * L * (B + 1) does not fit the index arithmetic         */
#define SPDY_DP_ERR_LAUNCH (-9)    /* the HIP runtime refused a launch (see hipGetLastError)    */

/* Bytes of device workspace spdy_dp_solve_batched / spdy_dp_fill need for these sizes, or 0 if
 * the sizes are invalid (see the status codes above).  The workspace holds the per-cell level
 * record P of Alg. 1 (one byte per (k, l, t), rows padded to a multiple of 64 buckets), the
 * final time t* per candidate, and -- when two D rows of B + 1 floats do not fit the 160 KB
 * of LDS of one compute unit -- two D rows per candidate. */
size_t spdy_dp_workspace_bytes(int K, int L, int S, int B);

/* Solve all K candidates: the whole of Alg. 1 (table fill, final argmin over t, walk back).
 *   tau      in  int32 [L][S]     times in buckets, >= 0, shared by all candidates
 *   err      in  fp32  [K][L][S]  errors, finite or +inf
 *   profile  out int16 [K][L]     chosen level per layer in [0, S), or -1 if infeasible
 *   cost     out fp32  [K]        optimal error, +inf if infeasible
 * Equivalent to spdy_dp_fill followed by spdy_dp_backtrace on the same stream. */
int spdy_dp_solve_batched(const int32_t *tau, const float *err, int K, int L, int S, int B,
                          int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                          void *stream);

/* First part of Alg. 1: fills the tables layer by layer (Eq. 2-3), records the chosen level of
 * every cell in the workspace, and takes the final argmin over t <= B.  Writes cost[k] and keeps
 * t*[k] in the workspace for spdy_dp_backtrace. */
int spdy_dp_fill(const int32_t *tau, const float *err, int K, int L, int S, int B, float *cost,
                 void *workspace, size_t workspace_bytes, void *stream);

/* Last loop of Alg. 1: walks the recorded levels back from (L-1, t*[k]) and writes profile[k].
 * `workspace` must be the one a spdy_dp_fill call with the same K, L, S, B and tau has filled
 * earlier on the same stream (or on a stream already synchronised with it). */
int spdy_dp_backtrace(const int32_t *tau, int K, int L, int S, int B, int16_t *profile,
                      const void *workspace, size_t workspace_bytes, void *stream);

/* Debug/test accessors describing the workspace layout for given sizes: byte offset of the
 * level record P, its row pitch in bytes (P[k][l][t] is at offset + ((k*L + l)*pitch + t)), and
 * the byte offset of the int32 t*[K] array.  Return SPDY_DP_OK or a size error. */
int spdy_dp_workspace_layout(int K, int L, int S, int B, size_t *choice_offset,
                             size_t *choice_pitch, size_t *tstar_offset);

/* Static, human-readable text for a status code. */
const char *spdy_dp_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPDY_DP_H */
