/*
 * CPU oracle for the two-stage depth-compression dynamic program.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the HIP path and
 * must never be called from it.  Build: gcc -O2 -ffp-contract=off (no
 * fast-math), see oracle/build.py.
 *
 * What it follows
 *   oracle_stage1      Algorithm 1 ("Finding Optimal Latency with DP"),
 *                      definitions Eq. 5a/5b, base case T_opt[k,k] = 0.
 *   oracle_relax_row   one row l of Algorithm 2 ("Solving the Surrogate
 *   oracle_stage2      Objective with DP"), recurrence Eq. 7a-7c, table D of
 *                      the footnote in Section 4.4 (called M here).
 *   oracle_backtrack   the set updates in the last two lines of Algorithm 2's
 *                      loop body and in Algorithm 1's if-branch, unrolled from
 *                      (L, T0) back to layer 0 through stored arg-max / arg-min
 *                      pointers instead of stored sets.
 *
 * Readings of the paper taken here (each is listed in the design notes):
 *   - budgets are inclusive: row l, column t covers total latency <= t; the
 *     paper's strict "< t" column is this table shifted by one column;
 *   - a cell that no feasible (A, S) reaches holds -inf instead of the
 *     paper's untouched 0, so the side constraint
 *     T_opt[0,k'] + T_opt[k',l] <= t of Algorithm 2 is carried by the values
 *     themselves (a -inf candidate never wins);
 *   - arg-min of Algorithm 1 takes the lowest m', arg-max of Algorithm 2 the
 *     lowest k';
 *   - "not mergeable" is T = DPC_INF = 2^30 - 1 and sums saturate there;
 *   - the objective is accumulated in IEEE binary32, one rounded add per
 *     block, left to right along the chain 0 -> a_1 -> ... -> l.
 *
 * Layout: every table is row-major with leading dimension ld = L + 1 for
 * (L+1) x (L+1) tables and P for (L+1) x P tables.  Only entries [i][j] with
 * i < j of T and I are read.
 *
 * Pins: tests/test_oracle_*.py (exhaustive enumeration in dpc_brute.c,
 * shortest paths, the worked example of Fig. 2, closed forms, invariants, a
 * literal set-carrying transcription of the recurrences).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define DPC_INF 0x3FFFFFFF
#define DPC_NOARG 0xFF

static int32_t sat_add(int32_t a, int32_t b)
{
    int64_t s = (int64_t)a + (int64_t)b;
    return s >= DPC_INF ? DPC_INF : (int32_t)s;
}

/* Algorithm 1.  T, Topt: int32 [L+1][L+1]; split: uint8 [L+1][L+1].
 * split[k][l] is the arg-min m of the algorithm: m == k means the layers
 * k+1..l form one merged block (S_opt[k,l] is empty); otherwise
 * S_opt[k,l] = S_opt[k,m] + {m}.  Entries with k >= l: Topt = 0 on the
 * diagonal (the base case) and below it, split = 0. */
void oracle_stage1(int32_t L, const int32_t *T, int32_t *Topt, uint8_t *split)
{
    const int32_t ld = L + 1;
    for (int32_t k = 0; k <= L; ++k)
        for (int32_t l = 0; l <= L; ++l) {
            Topt[k * ld + l] = 0;
            split[k * ld + l] = 0;
        }
    for (int32_t l = 1; l <= L; ++l) {
        for (int32_t k = 0; k < l; ++k) {
            int32_t best = DPC_INF;
            int32_t m = k;
            for (int32_t mp = k; mp < l; ++mp) {
                int32_t c = sat_add(Topt[k * ld + mp], T[mp * ld + l]);
                if (c < best) {
                    best = c;
                    m = mp;
                }
            }
            Topt[k * ld + l] = best;
            split[k * ld + l] = (uint8_t)m;
        }
    }
}

/* One row of Algorithm 2: fills M[j][0..P) and K[j][0..P) from rows i < j.
 * M: float [L+1][P]; K: uint8 [L+1][P] (may be NULL). */
void oracle_relax_row(int32_t L, int32_t P, int32_t j, const int32_t *Topt,
                      const float *I, float *M, uint8_t *K)
{
    const int32_t ld = L + 1;
    for (int32_t t = 0; t < P; ++t) {
        float best = -INFINITY;
        uint8_t arg = DPC_NOARG;
        for (int32_t i = 0; i < j; ++i) {
            int32_t w = Topt[i * ld + j];
            if (w <= t) {
                float c = M[(size_t)i * P + (t - w)] + I[i * ld + j];
                if (c > best) {
                    best = c;
                    arg = (uint8_t)i;
                }
            }
        }
        M[(size_t)j * P + t] = best;
        if (K)
            K[(size_t)j * P + t] = arg;
    }
}

/* Algorithm 2 for every budget t in [0, P) at once.  Row 0 is the base case
 * (no layer, objective +0 for every budget, A = S = empty). */
void oracle_stage2(int32_t L, int32_t P, const int32_t *Topt, const float *I,
                   float *M, uint8_t *K)
{
    for (int32_t t = 0; t < P; ++t) {
        M[t] = 0.0f;
        if (K)
            K[t] = DPC_NOARG;
    }
    for (int32_t j = 1; j <= L; ++j)
        oracle_relax_row(L, P, j, Topt, I, M, K);
}

/* Recover A[L,T0] and S[L,T0].  A, S: int32 [L] (ascending on return);
 * returns 0 and fills lengths, objective and latency, or returns 1 for a
 * budget no (A, S) meets (lengths -1, objective -inf, latency -1).
 * K == NULL: the arg-max is found again from M (lowest i that reproduces the
 * stored cell bit for bit). */
int32_t oracle_backtrack(int32_t L, int32_t P, const int32_t *Topt,
                         const uint8_t *split, const float *I, const float *M,
                         const uint8_t *K, int32_t T0, int32_t *A,
                         int32_t *A_len, int32_t *S, int32_t *S_len, float *obj,
                         int32_t *lat)
{
    const int32_t ld = L + 1;
    float top = M[(size_t)L * P + T0];
    if (top == -INFINITY) {
        *A_len = -1;
        *S_len = -1;
        *obj = -INFINITY;
        *lat = -1;
        return 1;
    }
    int32_t na = 0, ns = 0, total = 0;
    int32_t j = L, t = T0;
    while (j > 0) {
        int32_t i;
        if (K) {
            i = K[(size_t)j * P + t];
        } else {
            float want = M[(size_t)j * P + t];
            for (i = 0; i < j; ++i) {
                int32_t w = Topt[i * ld + j];
                if (w <= t) {
                    float c = M[(size_t)i * P + (t - w)] + I[i * ld + j];
                    if (c == want)
                        break;
                }
            }
        }
        /* S_opt[i,j]: follow the arg-min pointers down from j to i. */
        int32_t l = j;
        for (;;) {
            int32_t m = split[i * ld + l];
            if (m == i)
                break;
            S[ns++] = m;
            l = m;
        }
        if (i > 0) {
            A[na++] = i;
            S[ns++] = i;
        }
        total += Topt[i * ld + j];
        t -= Topt[i * ld + j];
        j = i;
    }
    /* collected from high to low: reverse into ascending order */
    for (int32_t a = 0, b = na - 1; a < b; ++a, --b) {
        int32_t x = A[a]; A[a] = A[b]; A[b] = x;
    }
    for (int32_t a = 0, b = ns - 1; a < b; ++a, --b) {
        int32_t x = S[a]; S[a] = S[b]; S[b] = x;
    }
    *A_len = na;
    *S_len = ns;
    *obj = top;
    *lat = total;
    return 0;
}
