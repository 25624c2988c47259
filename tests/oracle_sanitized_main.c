/*
 * Driver that runs the oracle's C routines under AddressSanitizer and UndefinedBehaviorSanitizer.
 *
 * TEST INFRASTRUCTURE ONLY (CPU).  tests/test_oracle_sanitized.py compiles this file together
 * with oracle/spdy_dp_ref.c and oracle/brute_force.c with -fsanitize=address,undefined, feeds it
 * instances on stdin and compares what it prints with the results of the ordinary build; any
 * out-of-bounds access, use of freed memory, leak or undefined arithmetic aborts the run.
 *
 * Input, whitespace separated, repeated until end of file:
 *     K L S B brute   tau[L*S] (int)   err[K*L*S] (fp32 bit patterns, hex)
 * Output per instance: one line "status", then per candidate "cost_bits level..." and, for
 * candidate 0, "D" and "P" rows of the full tables; with brute = 1 also the enumerator's
 * "cost_bits time n_best level...".
 */
#include <inttypes.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int spdy_dp_solve_ref(const int32_t *tau, const float *err, int K, int L, int S, int B,
                      int16_t *profile, float *cost);
int spdy_dp_solve_sens_ref(const int32_t *tau, const float *c, const float *w, int K, int L, int S,
                           int B, int16_t *profile, float *cost);
int spdy_dp_tables_ref(const int32_t *tau, const float *err, int L, int S, int B, float *D,
                       int32_t *P, int16_t *profile, float *cost);
int spdy_brute_force(const int32_t *tau, const float *err, int L, int S, int64_t B,
                     int16_t *best_profile, float *best_cost, int64_t *best_time, int64_t *n_best);

static uint32_t bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return u;
}

int main(void)
{
    int K, L, S, B, brute;
    while (scanf("%d %d %d %d %d", &K, &L, &S, &B, &brute) == 5) {
        const size_t cols = (size_t)B + 1;
        int32_t *tau = malloc((size_t)L * S * sizeof *tau);
        float *err = malloc((size_t)K * L * S * sizeof *err);
        int16_t *profile = malloc((size_t)K * L * sizeof *profile);
        float *cost = malloc((size_t)K * sizeof *cost);
        float *D = malloc((size_t)L * cols * sizeof *D);
        int32_t *P = malloc((size_t)L * cols * sizeof *P);
        if (!tau || !err || !profile || !cost || !D || !P)
            return 3;
        for (size_t i = 0; i < (size_t)L * S; ++i)
            if (scanf("%" SCNd32, &tau[i]) != 1)
                return 2;
        for (size_t i = 0; i < (size_t)K * L * S; ++i) {
            uint32_t u;
            if (scanf("%" SCNx32, &u) != 1)
                return 2;
            memcpy(&err[i], &u, sizeof u);
        }
        const int st = spdy_dp_solve_ref(tau, err, K, L, S, B, profile, cost);
        printf("status %d\n", st);
        if (st == 0) {
            for (int k = 0; k < K; ++k) {
                printf("%08" PRIx32, bits(cost[k]));
                for (int l = 0; l < L; ++l)
                    printf(" %d", profile[(size_t)k * L + l]);
                printf("\n");
            }
            int16_t *p0 = malloc((size_t)L * sizeof *p0);
            float c0;
            if (!p0 || spdy_dp_tables_ref(tau, err, L, S, B, D, P, p0, &c0) != 0)
                return 4;
            for (int l = 0; l < L; ++l) {
                printf("D");
                for (size_t t = 0; t < cols; ++t)
                    printf(" %08" PRIx32, bits(D[(size_t)l * cols + t]));
                printf("\nP");
                for (size_t t = 0; t < cols; ++t)
                    printf(" %d", P[(size_t)l * cols + t]);
                printf("\n");
            }
            free(p0);
            /* the sensitivity form on c = err[:, :, 0] and w = err[0, 0, :] (any finite numbers) */
            float *c = malloc((size_t)K * L * sizeof *c);
            if (!c)
                return 3;
            int finite = 1;
            for (int k = 0; k < K; ++k)
                for (int l = 0; l < L; ++l) {
                    c[(size_t)k * L + l] = err[((size_t)k * L + l) * S];
                    finite &= c[(size_t)k * L + l] - c[(size_t)k * L + l] == 0.0f;
                }
            for (int s = 0; s < S; ++s)
                finite &= err[s] - err[s] == 0.0f;
            if (finite) {
                const int st2 = spdy_dp_solve_sens_ref(tau, c, err, K, L, S, B, profile, cost);
                printf("sens %d", st2);
                for (int k = 0; k < K && st2 == 0; ++k)
                    printf(" %08" PRIx32, bits(cost[k]));
                printf("\n");
            }
            free(c);
        }
        if (brute) {
            int64_t bt, nb;
            float bc;
            const int sb = spdy_brute_force(tau, err, L, S, B, profile, &bc, &bt, &nb);
            printf("brute %d %08" PRIx32 " %" PRId64 " %" PRId64, sb, bits(bc), bt, nb);
            for (int l = 0; l < L; ++l)
                printf(" %d", profile[l]);
            printf("\n");
        }
        free(tau);
        free(err);
        free(profile);
        free(cost);
        free(D);
        free(P);
    }
    return 0;
}
