/*
 * Exhaustive enumeration for the extended objective (Appendix B of the paper,
 * the surrogate with end-activation flags and its budgeted maximisation).
 * TEST INFRASTRUCTURE ONLY: pins dpc_ext_oracle.c on tiny instances.
 *
 * brute_ext_objective: for the first l layers and every budget t in [0, P),
 *   max over A inside B inside {1..l-1}, S containing A, and the free flags
 *   d0 (at 0) and dl (at l) = out[t][dl], of the left-folded binary32 sum of
 *   I4[b_{j-1}, b_j, d(b_{j-1}), d(b_j)] along 0 -> B -> l, where d(x) = 1
 *   iff x is in A (interior) -- subject to the summed T along 0 -> S -> l
 *   being <= t.  Each interior position is in one of three states (absent,
 *   in B only, in A and B): 3^(l-1) pairs, and for each A the cheapest S
 *   containing A by enumerating all supersets.  out: float [P][2].
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define DPC_INF 0x3FFFFFFF
#define I4_AT(p, ld, k, l, a, b) ((p)[((((size_t)(k)) * (ld) + (l)) * 2 + (a)) * 2 + (b)])

static int32_t chain_latency_mask(int32_t ld, const int32_t *T, int32_t l, uint32_t smask)
{
    int64_t s = 0;
    int32_t prev = 0;
    for (int32_t x = 1; x <= l; ++x) {
        if (x == l || (smask >> (x - 1)) & 1u) {
            s += T[prev * ld + x];
            if (s >= DPC_INF)
                return DPC_INF;
            prev = x;
        }
    }
    return (int32_t)s;
}

void brute_ext_objective(int32_t ld, const int32_t *T, const float *I4, int32_t l, int32_t P,
                         float *out)
{
    const int32_t n = l - 1;                    /* interior positions 1..l-1 */
    for (int32_t t = 0; t < P; ++t)
        out[2 * t] = out[2 * t + 1] = -INFINITY;
    uint32_t total = 1;
    for (int32_t x = 0; x < n; ++x)
        total *= 3;
    for (uint32_t code = 0; code < total; ++code) {
        uint32_t amask = 0, bmask = 0, c = code;
        for (int32_t x = 0; x < n; ++x) {
            uint32_t st = c % 3;
            c /= 3;
            if (st >= 1)
                bmask |= 1u << x;
            if (st == 2)
                amask |= 1u << x;
        }
        /* cheapest S containing A */
        int32_t lat = DPC_INF;
        for (uint32_t sm = 0; sm < (1u << n); ++sm) {
            if ((sm & amask) != amask)
                continue;
            int32_t v = chain_latency_mask(ld, T, l, sm);
            if (v < lat)
                lat = v;
        }
        if (lat >= P)
            continue;
        for (int32_t d0 = 0; d0 < 2; ++d0)
            for (int32_t dl = 0; dl < 2; ++dl) {
                float acc = 0.0f;
                int32_t prev = 0, pflag = d0;
                for (int32_t x = 1; x <= l; ++x) {
                    if (x == l || (bmask >> (x - 1)) & 1u) {
                        int32_t flag = x == l ? dl : (int32_t)((amask >> (x - 1)) & 1u);
                        acc = acc + I4_AT(I4, ld, prev, x, pflag, flag);
                        prev = x;
                        pflag = flag;
                    }
                }
                for (int32_t t = lat; t < P; ++t)
                    if (acc > out[2 * t + dl])
                        out[2 * t + dl] = acc;
            }
    }
}
