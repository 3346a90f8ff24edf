/*
 * CPU oracle for the layer-by-layer plan-search dynamic program.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, serial, obviously-correct
 * statement of what the GPU library must compute.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code with the
 * HIP path and must never be used as a fallback by it.
 *
 * What it computes (paper section 3.3, "Dynamic Programming Search", Eq. 1,
 * with the readings listed below): for a stage of L layers, S candidate
 * strategies per layer and a memory budget of E units, the minimum over all
 * plans p in {0..S-1}^L with sum_l m(l, p_l) <= E of
 *
 *     sum_l c(l, p_l)  +  sum_{l>=1} R_{r_idx[l]}(p_{l-1}, p_l)
 *
 * together with one minimising plan.  The paper's optimal-substructure
 * argument (same section) is what makes the layer recurrence below exact.
 *
 * Readings where the paper's text is silent or inconsistent:
 *  - Eq. 1 is written with a two-index state C(L, E) although its transition
 *    term R(L, S_i, S_j) depends on the former layer's strategy.  The state
 *    here carries that strategy: C[l][e][s] = best time of layers 0..l using
 *    at most e memory units with layer l on strategy s.
 *  - R is indexed R[former layer's strategy][this layer's strategy]; it may
 *    be asymmetric and may have a non-zero diagonal.
 *  - "C(0, .) = 0": before the first layer nothing has been spent, so the
 *    first layer pays c(0, s) and no transition cost.  Feasibility is
 *    sum m <= E (inclusive).
 *  - "at most e" semantics: C is non-increasing in e.
 *  - Infinity (budget exceeded, the paper's Out-Of-Memory outcome in Alg. 1)
 *    is GALV_ORACLE_INF = 2^62; it never takes part in an addition.
 *  - Ties: the lowest former-strategy index wins every inner minimum (scan in
 *    ascending order, replace only on strictly smaller) and the lowest
 *    last-layer index wins the final minimum.
 *  - Unreachable cells hold INF and back-pointer -1; so do all cells of
 *    layer 0 (back-pointer only).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GALV_ORACLE_INF ((int64_t)1 << 62)

/*
 * One instance.  All pointers are host memory.
 *   c      [L][S]       execution time of layer l under strategy s, >= 0
 *   m      [L][S]       memory units of layer l under strategy s, >= 0
 *   R      [nR][S][S]   transformation cost, R[k][s_prev][s_cur] >= 0
 *   r_idx  [L] or NULL  matrix used between layer l-1 and l (NULL: matrix 0)
 *   budget              E, >= 0
 * Outputs:
 *   best_cost           optimum, or GALV_ORACLE_INF when no plan fits
 *   best_last           strategy of layer L-1 in the returned plan, or -1
 *   plan   [L]          the plan, all -1 when none fits
 *   C_last [budget+1][S] or NULL   last layer's table row by row (e major)
 *   bp     [L][budget+1][S] or NULL  back-pointers (former layer's strategy)
 *   n_tied or NULL      number of table cells (l >= 1) whose minimum is
 *                       attained by two or more finite candidates
 * Returns 0, or -1 on bad arguments, -2 when out of host memory.
 */
int galv_oracle_solve(int32_t L, int32_t S, int32_t nR,
                      const int64_t *c, const int32_t *m, const int64_t *R,
                      const int32_t *r_idx, int32_t budget,
                      int64_t *best_cost, int32_t *best_last, int32_t *plan,
                      int64_t *C_last, int32_t *bp, int64_t *n_tied)
{
    if (L < 1 || S < 1 || nR < 1 || budget < 0 || !c || !m || !R ||
        !best_cost || !best_last || !plan)
        return -1;

    const int64_t W = (int64_t)budget + 1;          /* table columns e = 0..E */
    int64_t *prev = malloc((size_t)(W * S) * sizeof(int64_t));
    int64_t *cur = malloc((size_t)(W * S) * sizeof(int64_t));
    int32_t *bp_own = NULL;
    if (!bp) {
        bp_own = malloc((size_t)((int64_t)L * W * S) * sizeof(int32_t));
        bp = bp_own;
    }
    if (!prev || !cur || !bp) {
        free(prev); free(cur); free(bp_own);
        return -2;
    }
    int64_t tied = 0;

    /* Layer 0: no former layer, hence no transition cost. */
    for (int64_t e = 0; e < W; ++e)
        for (int32_t s = 0; s < S; ++s) {
            prev[e * S + s] = ((int64_t)m[s] <= e) ? c[s] : GALV_ORACLE_INF;
            bp[e * S + s] = -1;
        }

    /* Layers 1..L-1: Eq. 1 with the former strategy in the state. */
    for (int32_t l = 1; l < L; ++l) {
        const int32_t k = r_idx ? r_idx[l] : 0;
        if (k < 0 || k >= nR) {
            free(prev); free(cur); free(bp_own);
            return -1;
        }
        const int64_t *Rl = R + (int64_t)k * S * S;
        int32_t *bpl = bp + (int64_t)l * W * S;
        for (int64_t e = 0; e < W; ++e)
            for (int32_t s = 0; s < S; ++s) {
                const int64_t ep = e - (int64_t)m[(int64_t)l * S + s];
                int64_t best = GALV_ORACLE_INF;
                int32_t arg = -1;
                int ties_here = 0;
                if (ep >= 0) {
                    for (int32_t sp = 0; sp < S; ++sp) {
                        const int64_t before = prev[ep * S + sp];
                        if (before == GALV_ORACLE_INF)
                            continue;
                        const int64_t cand = before + Rl[(int64_t)sp * S + s];
                        if (arg < 0 || cand < best) {
                            best = cand;
                            arg = sp;
                            ties_here = 0;
                        } else if (cand == best) {
                            ties_here = 1;
                        }
                    }
                }
                cur[e * S + s] = (arg < 0) ? GALV_ORACLE_INF
                                           : best + c[(int64_t)l * S + s];
                bpl[e * S + s] = arg;
                tied += ties_here;
            }
        int64_t *t = prev; prev = cur; cur = t;
    }

    /* Final minimum at the full budget, lowest index first. */
    int64_t opt = GALV_ORACLE_INF;
    int32_t last = -1;
    for (int32_t s = 0; s < S; ++s) {
        const int64_t v = prev[(int64_t)budget * S + s];
        if (v != GALV_ORACLE_INF && (last < 0 || v < opt)) {
            opt = v;
            last = s;
        }
    }
    *best_cost = opt;
    *best_last = last;

    /* Walk the back-pointers from the last layer to the first. */
    for (int32_t l = 0; l < L; ++l)
        plan[l] = -1;
    if (last >= 0) {
        int64_t e = budget;
        int32_t s = last;
        for (int32_t l = L - 1; l >= 1; --l) {
            plan[l] = s;
            const int32_t sp = bp[((int64_t)l * W + e) * S + s];
            e -= (int64_t)m[(int64_t)l * S + s];
            s = sp;
        }
        plan[0] = s;
    }

    if (C_last)
        memcpy(C_last, prev, (size_t)(W * S) * sizeof(int64_t));
    if (n_tied)
        *n_tied = tied;
    free(prev); free(cur); free(bp_own);
    return 0;
}

/* Value of "infinity", so that bindings need not repeat the constant. */
int64_t galv_oracle_inf(void) { return GALV_ORACLE_INF; }
