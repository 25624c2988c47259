/*
 * CPU oracle for the constrained layer-wise compression dynamic program.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is
 * checked against.  It shares no code with the GPU path, is single-threaded, and nothing in the
 * product may call it.
 *
 * What it computes (Sec. 3.1, Eq. 1): for every candidate k, levels s_1..s_L minimising
 * sum_l e_l^{s_l} subject to sum_l t_l^{s_l} <= T, with integer times, T = B buckets (Sec. 3.2).
 * How (Sec. 3.2, Eq. 2-3; App. A, Alg. 1): bottom-up dynamic programming over a cost matrix D
 * and a choice matrix P, both L x (T+1); D[l][t] is the least error of the first l layers that
 * take exactly time t.  The loops below keep the algorithm's nesting (layer, level, time) and
 * its names.
 *
 * Where the text leaves a choice open, this file takes the following readings:
 *  - numbers: D is fp32, one rounded add per update, layers accumulated in order 1..L;
 *    subnormals are kept (no flush-to-zero);
 *  - levels are visited in ascending index and an update needs a strictly smaller value, so the
 *    smallest level index wins a tie (the strict "<" is the algorithm's);
 *  - the inner time loop starts at t = t_l^s (so a prefix of time 0 can be extended); the
 *    algorithm prints t_l^s + 1, which never matters when every layer takes at least one bucket
 *    and would wrongly forbid zero-time prefixes otherwise;
 *  - a level whose time exceeds T is skipped (also in the first layer, where the algorithm
 *    indexes D[1][t_1^s] unguarded);
 *  - the final "argmin_t D[L][t]" returns the smallest such t;
 *  - if no profile meets the budget the candidate gets cost +inf and profile -1 (not an error);
 *  - err may be +inf (a forbidden level) or negative; NaN and -inf are rejected, and so is a
 *    negative time.
 *
 * Pinned (tests, CPU only) by exhaustive enumeration of Eq. 1 on small instances, by the 0/1
 * knapsack reduction, by closed forms (S = 1, L = 1, all times 0), by a hand-worked instance and
 * by invariants (budget met, monotone in B, dense profile when the budget allows it, re-summed
 * cost, scaling by powers of two).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

enum {
    REF_OK = 0,
    REF_ERR_NULL = -1,
    REF_ERR_DIM = -2,
    REF_ERR_LEVELS = -3,  /* S does not fit the int16 profile */
    REF_ERR_NEG_TIME = -6,
    REF_ERR_BAD_ERR = -7,
    REF_ERR_NOMEM = -8
};

/* Alg. 1 for one candidate.  t: [L][S] times, e: [L][S] errors, D: [L][T+1], P: [L][T+1].
 * Returns the optimal error (or +inf) and writes the chosen levels (or -1) to profile[L]. */
static float alg1(const int32_t *t, const float *e, int L, int S, int T, float *D, int32_t *P,
                  int16_t *profile)
{
    const size_t W = (size_t)T + 1;

    /* D <- L x (T+1) filled with inf; P <- L x (T+1) (no choice yet) */
    for (size_t i = 0; i < (size_t)L * W; ++i) {
        D[i] = INFINITY;
        P[i] = -1;
    }

    /* first layer: place e_1^s at exactly t_1^s, first smallest value wins */
    for (int s = 0; s < S; ++s) {
        const int32_t ts = t[s];
        if (ts > T)
            continue;
        if (e[s] < D[ts]) {
            D[ts] = e[s];
            P[ts] = s;
        }
    }

    /* layers 2..L */
    for (int l = 1; l < L; ++l) {
        const float *Dprev = D + (size_t)(l - 1) * W;
        float *Dl = D + (size_t)l * W;
        int32_t *Pl = P + (size_t)l * W;
        for (int s = 0; s < S; ++s) {
            const int32_t ts = t[(size_t)l * S + s];
            const float es = e[(size_t)l * S + s];
            for (int64_t tt = ts; tt <= T; ++tt) {
                const float v = es + Dprev[tt - ts];
                if (v < Dl[tt]) {
                    Dl[tt] = v;
                    Pl[tt] = s;
                }
            }
        }
    }

    /* t <- argmin_t D[L][t], smallest t among equals */
    const float *DL = D + (size_t)(L - 1) * W;
    int64_t tb = 0;
    for (int64_t tt = 1; tt <= T; ++tt)
        if (DL[tt] < DL[tb])
            tb = tt;
    const float best = DL[tb];
    if (!(best < INFINITY)) {
        for (int l = 0; l < L; ++l)
            profile[l] = -1;
        return INFINITY;
    }

    /* walk the choices back from layer L to layer 1 */
    for (int l = L - 1; l >= 0; --l) {
        const int32_t s = P[(size_t)l * W + (size_t)tb];
        profile[l] = (int16_t)s;
        tb -= t[(size_t)l * S + s];
    }
    return best;
}

static int check_inputs(const int32_t *tau, const float *err, int K, int L, int S, int B)
{
    if (!tau || !err)
        return REF_ERR_NULL;
    if (K <= 0 || L <= 0 || S <= 0 || B < 0)
        return REF_ERR_DIM;
    if (S > 32767)
        return REF_ERR_LEVELS;
    for (size_t i = 0; i < (size_t)L * S; ++i)
        if (tau[i] < 0)
            return REF_ERR_NEG_TIME;
    for (size_t i = 0; i < (size_t)K * L * S; ++i)
        if (isnan(err[i]) || (isinf(err[i]) && err[i] < 0))
            return REF_ERR_BAD_ERR;
    return REF_OK;
}

/* Solve K candidates that share one timing table.  All pointers are host pointers.
 * tau int32[L][S], err fp32[K][L][S], profile int16[K][L], cost fp32[K]. */
int spdy_dp_solve_ref(const int32_t *tau, const float *err, int K, int L, int S, int B,
                      int16_t *profile, float *cost)
{
    if (!profile || !cost)
        return REF_ERR_NULL;
    int st = check_inputs(tau, err, K, L, S, B);
    if (st != REF_OK)
        return st;
    const size_t W = (size_t)B + 1;
    float *D = (float *)malloc((size_t)L * W * sizeof(float));
    int32_t *P = (int32_t *)malloc((size_t)L * W * sizeof(int32_t));
    if (!D || !P) {
        free(D);
        free(P);
        return REF_ERR_NOMEM;
    }
    for (int k = 0; k < K; ++k)
        cost[k] = alg1(tau, err + (size_t)k * L * S, L, S, B, D, P, profile + (size_t)k * L);
    free(D);
    free(P);
    return REF_OK;
}

/* Error tables of the form of Eq. 4: err[k][l][s] = c[k][l] * w[s] (sensitivity of the layer times
 * a fixed weight of the level), each product ONE rounded fp32 multiply; then Alg. 1 as above.
 * c fp32[K][L], w fp32[S], both finite. */
int spdy_dp_solve_sens_ref(const int32_t *tau, const float *c, const float *w, int K, int L, int S,
                           int B, int16_t *profile, float *cost)
{
    if (!tau || !c || !w || !profile || !cost)
        return REF_ERR_NULL;
    if (K <= 0 || L <= 0 || S <= 0 || B < 0)
        return REF_ERR_DIM;
    float *e = (float *)malloc((size_t)L * S * sizeof(float));
    if (!e)
        return REF_ERR_NOMEM;
    int st = REF_OK;
    for (int k = 0; k < K && st == REF_OK; ++k) {
        for (int l = 0; l < L; ++l)
            for (int s = 0; s < S; ++s) {
                const float prod = c[(size_t)k * L + l] * w[s];
                e[(size_t)l * S + s] = prod;
            }
        st = spdy_dp_solve_ref(tau, e, 1, L, S, B, profile + (size_t)k * L, cost + k);
    }
    free(e);
    return st;
}

/* Same as above for ONE candidate, also handing back the full matrices (caller-allocated,
 * D fp32[L][B+1], P int32[L][B+1] with -1 where no level was chosen). */
int spdy_dp_tables_ref(const int32_t *tau, const float *err, int L, int S, int B, float *D,
                       int32_t *P, int16_t *profile, float *cost)
{
    if (!D || !P || !profile || !cost)
        return REF_ERR_NULL;
    int st = check_inputs(tau, err, 1, L, S, B);
    if (st != REF_OK)
        return st;
    *cost = alg1(tau, err, L, S, B, D, P, profile);
    return REF_OK;
}
