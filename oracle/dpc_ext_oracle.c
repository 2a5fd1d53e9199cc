/*
 * CPU oracle for the extended solver: block importances that depend on whether
 * the activations at both ends of a block are kept (Appendix B of the paper,
 * "Extension on the Importance").
 *
 * TEST INFRASTRUCTURE ONLY, like dpc_oracle.c: slow, plain, shares no code
 * with the HIP path.
 *
 * What it follows
 *   oracle_ext_iopt       Algorithm 3 ("Finding Optimal Importance with DP"):
 *                         max-plus interval DP over chains of blocks whose
 *                         interior end points carry an identity activation.
 *   oracle_ext_dp         Algorithm 4 ("Solving the Extended Surrogate
 *                         Objective"): the budgeted chain DP of Algorithm 2
 *                         with the extra state a = "is the activation at l
 *                         kept" and the extra choice alpha' at the predecessor.
 *   oracle_ext_backtrack  the set updates of Algorithm 4 (A, S, B) and of
 *                         Algorithms 1 and 3 (S_opt, B_opt), unrolled through
 *                         stored arg-max / arg-min pointers.
 *
 * Layout: I4 and Iopt are float [L+1][L+1][2][2], last two indices (a, b) =
 * (flag at the block's first end point k, flag at its last end point l);
 * bsplit uint8 likewise.  D is float [L+1][P][2] here (the HIP library stores
 * the same numbers as rows 2l+a of a table with 2L+3 rows); Kx uint8 likewise,
 * Kx = 2k'+alpha' of the winning predecessor, DPC_NOARG where nothing reaches.
 *
 * Readings of the paper taken here (listed in the design notes):
 *   - Algorithm 3's arg-max over k <= m' < l is read with the m' = k term
 *     standing for the single block (k, l) with its own end flags,
 *     I[k,l,a,b]; the printed term I_opt[k,k,a,0] + I[k,l,0,b] would drop the
 *     flag a of a one-block chain.  The single block is tried first, then
 *     m' = k+1, ..., l-1 in ascending order; a candidate replaces the maximum
 *     only when strictly greater.
 *   - B_opt depends on the end flags (the listing writes B_opt[k,l]): one
 *     arg-max pointer per (k, l, a, b).
 *   - Algorithm 4 is Algorithm 2 with budgets read inclusively and -inf in
 *     unreachable cells, as in dpc_oracle.c.  Candidates are tried in
 *     ascending (k', alpha') order, strict improvement only.  D[0][t][a] = +0
 *     for both a: the flag at the network input is free, and combinations a
 *     caller wants to exclude carry -inf in I4 (as the algorithm's first
 *     lines do for positions whose original activation is, or is not, an
 *     identity).  The listing's last line (arg-max over a of A[L,T0,a]) is
 *     read as the arg-max of D[L,T0,a], lowest a on ties.
 *   - objective in IEEE binary32, one rounded add per block, left to right.
 *
 * Pins: tests/test_ext_oracle_pins.py (exhaustive enumeration in
 * dpc_ext_brute.c, reduction to Algorithm 2 when I4 ignores the flags,
 * invariants, re-scoring of the recovered sets).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define DPC_INF 0x3FFFFFFF
#define DPC_NOARG 0xFF

#define I4_AT(p, ld, k, l, a, b) ((p)[((((size_t)(k)) * (ld) + (l)) * 2 + (a)) * 2 + (b)])

/* Algorithm 3.  bsplit[k][l][a][b] = the arg-max m: m == k means the chain is
 * the single block (k, l); otherwise B_opt[k,l,a,b] = B_opt[k,m,a,0] + {m}.
 * Entries with k >= l: Iopt = +0, bsplit = 0. */
void oracle_ext_iopt(int32_t L, const float *I4, float *Iopt, uint8_t *bsplit)
{
    const int32_t ld = L + 1;
    for (size_t x = 0; x < (size_t)ld * ld * 4; ++x) {
        Iopt[x] = 0.0f;
        bsplit[x] = 0;
    }
    for (int32_t l = 1; l <= L; ++l)
        for (int32_t k = 0; k < l; ++k)
            for (int32_t a = 0; a < 2; ++a)
                for (int32_t b = 0; b < 2; ++b) {
                    float best = I4_AT(I4, ld, k, l, a, b);
                    int32_t m = k;
                    for (int32_t mp = k + 1; mp < l; ++mp) {
                        float c = I4_AT(Iopt, ld, k, mp, a, 0) + I4_AT(I4, ld, mp, l, 0, b);
                        if (c > best) {
                            best = c;
                            m = mp;
                        }
                    }
                    I4_AT(Iopt, ld, k, l, a, b) = best;
                    I4_AT(bsplit, ld, k, l, a, b) = (uint8_t)m;
                }
}

/* Algorithm 4 for every budget t in [0, P).  D: float [L+1][P][2],
 * Kx: uint8 [L+1][P][2] (may be NULL). */
void oracle_ext_dp(int32_t L, int32_t P, const int32_t *Topt, const float *Iopt,
                   float *D, uint8_t *Kx)
{
    const int32_t ld = L + 1;
    for (int32_t t = 0; t < P; ++t)
        for (int32_t a = 0; a < 2; ++a) {
            D[((size_t)0 * P + t) * 2 + a] = 0.0f;
            if (Kx)
                Kx[((size_t)0 * P + t) * 2 + a] = DPC_NOARG;
        }
    for (int32_t l = 1; l <= L; ++l)
        for (int32_t t = 0; t < P; ++t)
            for (int32_t a = 0; a < 2; ++a) {
                float best = -INFINITY;
                uint8_t arg = DPC_NOARG;
                for (int32_t kp = 0; kp < l; ++kp) {
                    int32_t w = Topt[kp * ld + l];
                    if (w > t)
                        continue;
                    for (int32_t al = 0; al < 2; ++al) {
                        float c = D[((size_t)kp * P + (t - w)) * 2 + al] +
                                  I4_AT(Iopt, ld, kp, l, al, a);
                        if (c > best) {
                            best = c;
                            arg = (uint8_t)(2 * kp + al);
                        }
                    }
                }
                D[((size_t)l * P + t) * 2 + a] = best;
                if (Kx)
                    Kx[((size_t)l * P + t) * 2 + a] = arg;
            }
}

/* Recover A, S and B for budget T0.  A, S, Bs: int32 [L] (ascending on
 * return).  Returns 0, or 1 when no solution meets the budget (lengths -1,
 * objective -inf, latency -1). */
int32_t oracle_ext_backtrack(int32_t L, int32_t P, const int32_t *Topt,
                             const uint8_t *split, const uint8_t *bsplit, const float *D,
                             const uint8_t *Kx, int32_t T0, int32_t *A, int32_t *A_len,
                             int32_t *S, int32_t *S_len, int32_t *Bs, int32_t *B_len,
                             float *obj, int32_t *lat, int32_t *a_last)
{
    const int32_t ld = L + 1;
    float d0 = D[((size_t)L * P + T0) * 2 + 0], d1 = D[((size_t)L * P + T0) * 2 + 1];
    int32_t a = d1 > d0 ? 1 : 0;               /* lowest a on ties */
    float top = a ? d1 : d0;
    if (top == -INFINITY) {
        *A_len = *S_len = *B_len = -1;
        *obj = -INFINITY;
        *lat = -1;
        *a_last = -1;
        return 1;
    }
    *a_last = a;
    int32_t na = 0, ns = 0, nb = 0, total = 0;
    int32_t l = L, t = T0;
    while (l > 0) {
        int32_t arg = Kx[((size_t)l * P + t) * 2 + a];
        int32_t k = arg >> 1, al = arg & 1;
        /* S_opt[k,l]: arg-min pointers of Algorithm 1 from l down to k */
        for (int32_t x = l;;) {
            int32_t m = split[k * ld + x];
            if (m == k)
                break;
            S[ns++] = m;
            x = m;
        }
        /* B_opt[k,l,al,a]: arg-max pointers of Algorithm 3; the chain to the
         * left of a split point m ends with flag 0 at m */
        for (int32_t x = l, bflag = a;;) {
            int32_t m = I4_AT(bsplit, ld, k, x, al, bflag);
            if (m == k)
                break;
            Bs[nb++] = m;
            x = m;
            bflag = 0;
        }
        if (k > 0) {
            if (al)
                A[na++] = k;
            S[ns++] = k;
            Bs[nb++] = k;
        }
        total += Topt[k * ld + l];
        t -= Topt[k * ld + l];
        l = k;
        a = al;
    }
#define REVERSE(v, n) for (int32_t x_ = 0, y_ = (n) - 1; x_ < y_; ++x_, --y_) { int32_t z_ = (v)[x_]; (v)[x_] = (v)[y_]; (v)[y_] = z_; }
    REVERSE(A, na)
    REVERSE(S, ns)
    REVERSE(Bs, nb)
    *A_len = na;
    *S_len = ns;
    *B_len = nb;
    *obj = top;
    *lat = total;
    return 0;
}
