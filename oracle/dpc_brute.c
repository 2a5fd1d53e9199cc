/*
 * Exhaustive enumeration for tiny L: the plain definitions that pin the
 * oracle in dpc_oracle.c.  TEST INFRASTRUCTURE ONLY; nothing here is a
 * dynamic program and nothing here is shared with dpc_oracle.c or with the
 * HIP path.
 *
 *   brute_topt      Eq. 5a: minimum over every S inside {k+1..l-1} of the
 *                   summed block latencies of the chain k -> S -> l.
 *   brute_objective Eq. 6 (the sub-problem of Eq. 4 for the first l layers),
 *                   inclusive budget: for every t in [0, P) the maximum over
 *                   all pairs A inside S inside {1..l-1} with chain latency
 *                   <= t of the summed block importances of 0 -> A -> l.
 *   brute_min_latency_given_A
 *                   Eq. 8 (Proposition 4.2): minimum chain latency over every
 *                   S that contains a given A.
 *
 * Importances are summed in binary32 from +0, left to right along the chain,
 * which is the order in which the recurrence of Eq. 7 accumulates them.
 * Latencies saturate at DPC_INF = 2^30 - 1 ("not mergeable").
 * Tables are row-major with leading dimension ld.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define DPC_INF 0x3FFFFFFF

/* chain latency of k -> (members of mask, bit (x-k-1) <-> index x) -> l */
static int32_t chain_latency(int32_t ld, const int32_t *T, int32_t k, int32_t l,
                             uint32_t mask)
{
    int64_t sum = 0;
    int32_t prev = k;
    for (int32_t x = k + 1; x <= l; ++x) {
        if (x == l || ((mask >> (x - k - 1)) & 1u)) {
            sum += T[prev * ld + x];
            if (sum >= DPC_INF)
                return DPC_INF;
            prev = x;
        }
    }
    return (int32_t)sum;
}

int32_t brute_topt(int32_t ld, const int32_t *T, int32_t k, int32_t l)
{
    if (k == l)
        return 0;
    int32_t best = DPC_INF;
    uint32_t n = 1u << (l - k - 1);
    for (uint32_t mask = 0; mask < n; ++mask) {
        int32_t c = chain_latency(ld, T, k, l, mask);
        if (c < best)
            best = c;
    }
    return best;
}

/* out[t], t in [0, P): best objective with latency <= t, -inf if none.
 * l - 1 <= 15 positions; 3^(l-1) pairs. */
void brute_objective(int32_t ld, const int32_t *T, const float *I, int32_t l,
                     int32_t P, float *out)
{
    for (int32_t t = 0; t < P; ++t)
        out[t] = -INFINITY;
    int32_t n = l - 1; /* free positions 1..l-1 */
    int32_t state[16]; /* 0: not in S, 1: in S only, 2: in A (and S) */
    for (int32_t x = 0; x < 16; ++x)
        state[x] = 0;
    for (;;) {
        uint32_t smask = 0, amask = 0;
        for (int32_t x = 0; x < n; ++x) {
            if (state[x] >= 1)
                smask |= 1u << x;
            if (state[x] == 2)
                amask |= 1u << x;
        }
        int32_t lat = chain_latency(ld, T, 0, l, smask);
        if (lat < P) {
            float obj = 0.0f;
            int32_t prev = 0;
            for (int32_t x = 1; x <= l; ++x) {
                if (x == l || ((amask >> (x - 1)) & 1u)) {
                    obj = obj + I[prev * ld + x];
                    prev = x;
                }
            }
            if (obj > out[lat])
                out[lat] = obj;
        }
        /* next base-3 counter value */
        int32_t x = 0;
        while (x < n && state[x] == 2)
            state[x++] = 0;
        if (x == n)
            break;
        state[x]++;
    }
    /* "latency <= t": running maximum over the exact-latency buckets */
    for (int32_t t = 1; t < P; ++t)
        if (out[t - 1] > out[t])
            out[t] = out[t - 1];
}

/* amask: bit (x-1) set <-> x in A, x in 1..l-1 */
int32_t brute_min_latency_given_A(int32_t ld, const int32_t *T, int32_t l,
                                  uint32_t amask)
{
    int32_t best = DPC_INF;
    uint32_t n = 1u << (l - 1);
    for (uint32_t smask = 0; smask < n; ++smask) {
        if ((smask & amask) != amask)
            continue;
        int32_t c = chain_latency(ld, T, 0, l, smask);
        if (c < best)
            best = c;
    }
    return best;
}
