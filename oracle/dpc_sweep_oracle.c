/*
 * CPU oracle for the steps around the solver in a hyper-parameter sweep.
 *
 * TEST INFRASTRUCTURE ONLY: the plain reference the GPU library is checked
 * against.  It shares no code with the HIP path and must never be called from
 * it.  Build: gcc -O2 -ffp-contract=off (no fast-math), see oracle/build.py.
 *
 * What it follows
 *   oracle_importance_shift   the normalisation of Appendix "Evaluating and
 *                             Normalizing the Importance": every block's
 *                             importance is lowered by alpha times the mean
 *                             importance of the blocks of size one.
 *   oracle_front              the budgets at which the optimum of Eq. 4
 *                             changes, read off the last row of Algorithm 2's
 *                             table: the (latency, objective) trade-off curve
 *                             that the sweeps over T0 in the experiments walk.
 *   oracle_front_queries      the points of the curves of a batch as a flat list
 *                             of (instance, budget) pairs, the budgets a sweep
 *                             over T0 has to recover sets for.
 *   oracle_chain_latency      the latency of a network merged at a given
 *                             ordered set (left side of the constraint in
 *                             Eq. 4 with the given set in place of S); with
 *                             the set A it is the "merged with A" curve of
 *                             the ablation on the ordered set to be merged.
 *
 * Readings taken here (listed in the design notes):
 *   - the set D of the normalisation is taken as the multiset of the FINITE
 *     entries I[i][i+1] (all four flag combinations when the table has flags):
 *     a block excluded from the DP by -inf has no accuracy change to average;
 *     an empty D means no shift;
 *   - the mean is accumulated in binary64 in ascending order of (i, flags),
 *     the product alpha * mean is rounded once to binary64, and each output is
 *     the binary32 rounding of the binary64 difference;
 *   - a point (t, M[L][t]) belongs to the trade-off curve when M[L][t] is
 *     finite and greater than M[L][t-1] (column -1 counts as -inf).
 *
 * Pins: tests/test_sweep_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define DPC_INF 0x3FFFFFFF

/* I_raw, I_out: float [L+1][L+1][F], F = 1 (plain table) or 4 (flags a, b).
 * Returns the mean of D (0 when D is empty). */
double oracle_importance_shift(int32_t L, int32_t F, const float *I_raw, float alpha,
                               float *I_out)
{
    const int32_t ld = L + 1;
    double sum = 0.0;
    int32_t count = 0;
    for (int32_t i = 0; i < L; ++i)
        for (int32_t f = 0; f < F; ++f) {
            float v = I_raw[((size_t)i * ld + (i + 1)) * F + f];
            if (isfinite(v)) {
                sum += (double)v;
                ++count;
            }
        }
    const double mean = count > 0 ? sum / (double)count : 0.0;
    const double shift = (double)alpha * mean;
    for (size_t x = 0; x < (size_t)ld * ld * F; ++x)
        I_out[x] = (float)((double)I_raw[x] - shift);
    return mean;
}

/* Mrow: the last row of the stage-2 table, float [P].  Writes at most cap
 * points (budget ascending) and returns how many there are in all. */
int32_t oracle_front(int32_t P, const float *Mrow, int32_t cap, int32_t *front_t,
                     float *front_obj)
{
    int32_t n = 0;
    float below = -INFINITY;
    for (int32_t t = 0; t < P; ++t) {
        float v = Mrow[t];
        if (v > below) {
            if (n < cap) {
                front_t[n] = t;
                front_obj[n] = v;
            }
            ++n;
        }
        below = v;
    }
    return n;
}

/* X: ascending members of [1, L-1], n of them (n < 0: no set, returns -1).
 * Sum of T along 0 -> X -> L, saturating at DPC_INF. */
int32_t oracle_chain_latency(int32_t L, const int32_t *T, int32_t n, const int32_t *X)
{
    if (n < 0)
        return -1;
    const int32_t ld = L + 1;
    int64_t total = 0;
    int32_t from = 0;
    for (int32_t x = 0; x <= n; ++x) {
        int32_t to = x < n ? X[x] : L;
        total += T[from * ld + to];
        if (total >= DPC_INF)
            total = DPC_INF;
        from = to;
    }
    return (int32_t)total;
}

/* front_t: int32 [B][cap], front_len: int32 [B] as written by oracle_front for
 * every instance (lengths may exceed cap: then cap points were stored).  Writes
 * at most qcap queries, instance by instance, budgets ascending, and returns
 * how many there are in all. */
int32_t oracle_front_queries(int32_t B, int32_t cap, const int32_t *front_t,
                             const int32_t *front_len, int32_t qcap, int32_t *q_inst,
                             int32_t *q_T0)
{
    int32_t n = 0;
    for (int32_t b = 0; b < B; ++b) {
        int32_t len = front_len[b] < cap ? front_len[b] : cap;
        for (int32_t k = 0; k < len; ++k) {
            if (n < qcap) {
                q_inst[n] = b;
                q_T0[n] = front_t[(size_t)b * cap + k];
            }
            ++n;
        }
    }
    return n;
}
