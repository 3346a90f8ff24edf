/*
 * Stand-alone driver for galv_oracle.c, meant to be built with
 *     gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all
 * and run by the CPU test-suite: it solves the instances it reads from stdin and prints
 * what the oracle returns, so that any out-of-bounds access, use of uninitialised
 * heap, signed overflow or misaligned access inside the oracle aborts the run.
 * TEST INFRASTRUCTURE ONLY; it holds none of the method's arithmetic.
 *
 * Input (text, whitespace separated), repeated until end of file:
 *     L S nR budget has_r_idx want_tables
 *     c[L*S]  m[L*S]  R[nR*S*S]  r_idx[L] (only when has_r_idx)
 * Output per instance, one line:
 *     rc best_cost best_last n_tied plan[0..L-1] sum(C_last mod 2^31) sum(bp + 1)
 * (the two sums only when want_tables, else 0 0).
 */
#include <inttypes.h>
#include <stdio.h>
#include <stdlib.h>

#include "galv_oracle.c"

int main(void)
{
    int32_t L, S, nR, budget, has_r_idx, want_tables;
    while (scanf("%" SCNd32 " %" SCNd32 " %" SCNd32 " %" SCNd32 " %" SCNd32 " %" SCNd32,
                 &L, &S, &nR, &budget, &has_r_idx, &want_tables) == 6) {
        const size_t ls = (size_t)L * S, rs = (size_t)nR * S * S, w = (size_t)budget + 1;
        int64_t *c = malloc(ls * sizeof *c), *R = malloc(rs * sizeof *R);
        int32_t *m = malloc(ls * sizeof *m), *r_idx = has_r_idx ? malloc((size_t)L * sizeof *r_idx) : NULL;
        int32_t *plan = malloc((size_t)L * sizeof *plan);
        int64_t *C_last = want_tables ? malloc(w * S * sizeof *C_last) : NULL;
        int32_t *bp = want_tables ? malloc((size_t)L * w * S * sizeof *bp) : NULL;
        if (!c || !R || !m || !plan || (has_r_idx && !r_idx) || (want_tables && (!C_last || !bp)))
            return 2;
        for (size_t i = 0; i < ls; ++i) if (scanf("%" SCNd64, &c[i]) != 1) return 3;
        for (size_t i = 0; i < ls; ++i) if (scanf("%" SCNd32, &m[i]) != 1) return 3;
        for (size_t i = 0; i < rs; ++i) if (scanf("%" SCNd64, &R[i]) != 1) return 3;
        for (int32_t i = 0; has_r_idx && i < L; ++i) if (scanf("%" SCNd32, &r_idx[i]) != 1) return 3;

        int64_t best_cost = -1, n_tied = -1;
        int32_t best_last = -2;
        const int rc = galv_oracle_solve(L, S, nR, c, m, R, r_idx, budget, &best_cost, &best_last,
                                         plan, C_last, bp, &n_tied);
        printf("%d %" PRId64 " %" PRId32 " %" PRId64, rc, best_cost, best_last, n_tied);
        for (int32_t l = 0; l < L; ++l) printf(" %" PRId32, plan[l]);
        int64_t sum_c = 0, sum_bp = 0;
        if (want_tables && rc == 0) {
            for (size_t i = 0; i < w * S; ++i) sum_c += C_last[i] % ((int64_t)1 << 31);
            for (size_t i = 0; i < (size_t)L * w * S; ++i) sum_bp += bp[i] + 1;
        }
        printf(" %" PRId64 " %" PRId64 "\n", sum_c, sum_bp);
        free(c); free(R); free(m); free(r_idx); free(plan); free(C_last); free(bp);
    }
    return 0;
}
