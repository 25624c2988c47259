/*
 * CPU oracle for the constrained layer-wise compression dynamic program.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is
 * checked against.  It shares no code with the GPU path, is single-threaded, and nothing in the
 * product may call it.
 *
 * What it computes (Sec. 3.1, Eq. 1): for every candidate k, one level per layer minimising the
 * summed error subject to the summed integer time staying within the budget of B buckets
 * (Sec. 3.2).  How (Sec. 3.2, Eq. 2-3; App. A, Alg. 1): dynamic programming over time.  With
 * least[l][t] = the least error of layers 0..l taking EXACTLY time t, Eq. 2 reads
 *
 *     least[l][t] = min over levels s of  least[l-1][t - tau[l][s]] + err[l][s],
 *
 * the answer is the smallest least[L-1][t] over t <= B, and the levels are recovered by walking
 * the per-cell choices back from that cell.
 *
 * Shape of this implementation.  Each cell is computed on its own: for a layer l and a time t,
 * the levels are tried in ascending index and a level replaces the running best only when its
 * value is strictly smaller (so the smallest level index wins a tie, as the strict "<" of Alg. 1
 * implies when levels are visited in ascending order).  For one cell this is the same sequence
 * of comparisons as a level-major sweep over the whole row, so both produce identical tables.
 * Only two rows of values are alive at a time (the row being built reads the previous row only);
 * the per-cell choices of all layers are kept for the walk back.  The first layer needs no
 * special case: Eq. 3 (layer 1 puts err[0][s] at time tau[0][s]) is Eq. 2 applied to a start row
 * that is reachable at time 0 only, with the value -0.0f there, because x + (-0.0f) returns x
 * bit for bit for every x (with +0.0f, an error of -0.0f would come out as +0.0f).
 *
 * Where the text leaves a choice open, this file takes the following readings:
 *  - numbers: values are fp32, one rounded add per (cell, level), layers accumulated in order
 *    0..L-1; subnormals are kept (no flush-to-zero);
 *  - the printed inner loop starts at t = t_l^s + 1; here a level applies from t = tau[l][s] on
 *    (t - tau >= 0), so a prefix of time 0 can be extended; the printed bound never matters when
 *    every layer takes at least one bucket and would wrongly forbid zero-time prefixes otherwise;
 *  - a level whose time exceeds the budget never applies (also in the first layer, which the
 *    printed algorithm indexes unguarded);
 *  - the final argmin over t returns the smallest such t;
 *  - if no profile meets the budget the candidate gets cost +inf and profile -1 (not an error);
 *  - err may be +inf (a forbidden level) or negative; NaN and -inf are rejected, and so is a
 *    negative time.
 *
 * Pinned (tests, CPU only) by exhaustive enumeration of Eq. 1 on small instances, by hand-worked
 * instances (unique optima, and tied optima under a binding budget), by the 0/1 knapsack
 * reduction, by an integer-programming routine, by closed forms (S = 1, L = 1, all times 0) and
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

#define NO_LEVEL (-1)

/* Scratch of one solve: two rows of values and the choices of every cell. */
struct scratch {
    float *row_a, *row_b;  /* [B + 1] each */
    int32_t *choice;       /* [L][B + 1], NO_LEVEL where nothing reaches the cell */
};

static int scratch_alloc(struct scratch *w, int L, int B)
{
    const size_t cols = (size_t)B + 1;
    w->row_a = (float *)malloc(cols * sizeof(float));
    w->row_b = (float *)malloc(cols * sizeof(float));
    w->choice = (int32_t *)malloc((size_t)L * cols * sizeof(int32_t));
    return (w->row_a && w->row_b && w->choice) ? REF_OK : REF_ERR_NOMEM;
}

static void scratch_free(struct scratch *w)
{
    free(w->row_a);
    free(w->row_b);
    free(w->choice);
}

/* One candidate.  tau [L][S], err [L][S]; writes profile[L] and returns the optimal error (+inf
 * and profile -1 when no profile meets the budget).  If all_rows is given it receives every row
 * of values, [L][B + 1]. */
static float solve_one(const int32_t *tau, const float *err, int L, int S, int B,
                       struct scratch *w, int16_t *profile, float *all_rows)
{
    const size_t cols = (size_t)B + 1;
    float *below = w->row_a;   /* values after the previous layer */
    float *here = w->row_b;    /* values after this layer */

    /* before any layer: time 0 is reachable at no cost, nothing else is */
    below[0] = -0.0f;
    for (size_t t = 1; t < cols; ++t)
        below[t] = INFINITY;

    for (int l = 0; l < L; ++l) {
        const int32_t *tau_l = tau + (size_t)l * S;
        const float *err_l = err + (size_t)l * S;
        int32_t *choice_l = w->choice + (size_t)l * cols;
        for (int64_t t = 0; t <= B; ++t) {
            float best = INFINITY;
            int32_t arg = NO_LEVEL;
            for (int s = 0; s < S; ++s) {
                const int64_t before = t - tau_l[s];   /* time left for layers 0..l-1 */
                if (before < 0)
                    continue;
                const float v = below[before] + err_l[s];
                if (v < best) {
                    best = v;
                    arg = s;
                }
            }
            here[t] = best;
            choice_l[t] = arg;
        }
        if (all_rows)
            for (size_t t = 0; t < cols; ++t)
                all_rows[(size_t)l * cols + t] = here[t];
        float *swap = below;
        below = here;
        here = swap;
    }

    /* smallest time among the cells of least value in the last row */
    int64_t t_best = 0;
    for (int64_t t = 1; t <= B; ++t)
        if (below[t] < below[t_best])
            t_best = t;
    const float cost = below[t_best];
    if (!(cost < INFINITY)) {
        for (int l = 0; l < L; ++l)
            profile[l] = -1;
        return INFINITY;
    }

    /* recover the levels from the last layer down */
    int64_t t = t_best;
    for (int l = L - 1; l >= 0; --l) {
        const int32_t s = w->choice[(size_t)l * cols + (size_t)t];
        profile[l] = (int16_t)s;
        t -= tau[(size_t)l * S + s];
    }
    return cost;
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
    struct scratch w;
    st = scratch_alloc(&w, L, B);
    if (st == REF_OK)
        for (int k = 0; k < K; ++k)
            cost[k] = solve_one(tau, err + (size_t)k * L * S, L, S, B, &w,
                                profile + (size_t)k * L, NULL);
    scratch_free(&w);
    return st;
}

/* Error tables of the form of Eq. 4: err[k][l][s] = c[k][l] * w[s] (sensitivity of the layer times
 * a fixed weight of the level), each product ONE rounded fp32 multiply; then the solve above.
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

/* The solve for ONE candidate, also handing back the full tables (caller-allocated):
 * D fp32[L][B+1] = least[l][t], P int32[L][B+1] = the chosen level, -1 where none applies. */
int spdy_dp_tables_ref(const int32_t *tau, const float *err, int L, int S, int B, float *D,
                       int32_t *P, int16_t *profile, float *cost)
{
    if (!D || !P || !profile || !cost)
        return REF_ERR_NULL;
    int st = check_inputs(tau, err, 1, L, S, B);
    if (st != REF_OK)
        return st;
    struct scratch w;
    st = scratch_alloc(&w, L, B);
    if (st == REF_OK) {
        *cost = solve_one(tau, err, L, S, B, &w, profile, D);
        const size_t cells = (size_t)L * ((size_t)B + 1);
        for (size_t i = 0; i < cells; ++i)
            P[i] = w.choice[i];
    }
    scratch_free(&w);
    return st;
}
