/*
 * Exhaustive solver of the constrained problem (Sec. 3.1, Eq. 1) for tiny instances.
 *
 * TEST INFRASTRUCTURE ONLY.  It is the plain definition the dynamic program must reach: visit
 * every one of the S^L profiles, keep those whose total time is at most B, and take the one of
 * least total error.  Errors are summed in fp32 in layer order (e_1 first), the order the
 * dynamic program accumulates in; because a rounded add is monotone in its first operand, the
 * least such sum is bit-identical to the dynamic program's optimum.
 *
 * Among profiles of equal (error, time) the smallest under the key (s_L, s_{L-1}, .., s_1) is
 * returned, and the number of profiles attaining the best (error, time) pair is reported, so a
 * caller can tell when the optimum is unique.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* tau int32[L][S], err fp32[L][S].  Outputs: best_profile int16[L] (-1 if infeasible),
 * best_cost, best_time (-1 if infeasible), n_best = profiles with that (cost, time).
 * Returns 0, or -1 on bad arguments / S^L too large (> 2^40). */
int spdy_brute_force(const int32_t *tau, const float *err, int L, int S, int64_t B,
                     int16_t *best_profile, float *best_cost, int64_t *best_time,
                     int64_t *n_best)
{
    if (!tau || !err || !best_profile || !best_cost || !best_time || !n_best || L <= 0 || S <= 0 ||
        L > 64)
        return -1;
    double count = pow((double)S, (double)L);
    if (count > 1099511627776.0)
        return -1;

    int digit[64];
    int64_t ptime[65]; /* ptime[l+1] = time of layers 0..l under the current digits */
    float pcost[65];   /* pcost[l+1] = fp32 error sum of layers 0..l, left to right */
    memset(digit, 0, sizeof digit);

    int found = 0;
    float bc = INFINITY;
    int64_t bt = -1, nb = 0;
    int16_t bp[64];

    int from = 0; /* lowest layer whose digit changed since the last evaluation */
    for (;;) {
        for (int l = from; l < L; ++l) {
            const int32_t t = tau[(size_t)l * S + digit[l]];
            const float e = err[(size_t)l * S + digit[l]];
            ptime[l + 1] = (l == 0 ? 0 : ptime[l]) + t;
            pcost[l + 1] = (l == 0) ? e : pcost[l] + e;
        }
        const int64_t tt = ptime[L];
        const float cc = pcost[L];
        if (tt <= B && cc < INFINITY) {
            int better = 0, same = 0;
            if (!found || cc < bc || (cc == bc && tt < bt))
                better = 1;
            else if (cc == bc && tt == bt)
                same = 1;
            if (better) {
                found = 1;
                bc = cc;
                bt = tt;
                nb = 1;
                for (int l = 0; l < L; ++l)
                    bp[l] = (int16_t)digit[l];
            } else if (same) {
                ++nb;
                /* key: compare from the last layer down */
                for (int l = L - 1; l >= 0; --l) {
                    if (digit[l] != bp[l]) {
                        if (digit[l] < bp[l])
                            for (int j = 0; j < L; ++j)
                                bp[j] = (int16_t)digit[j];
                        break;
                    }
                }
            }
        }
        /* next profile: the last layer's digit moves fastest */
        int l = L - 1;
        while (l >= 0 && ++digit[l] == S) {
            digit[l] = 0;
            --l;
        }
        if (l < 0)
            break;
        from = l;
    }

    if (!found) {
        for (int l = 0; l < L; ++l)
            best_profile[l] = -1;
        *best_cost = INFINITY;
        *best_time = -1;
        *n_best = 0;
        return 0;
    }
    for (int l = 0; l < L; ++l)
        best_profile[l] = bp[l];
    *best_cost = bc;
    *best_time = bt;
    *n_best = nb;
    return 0;
}
