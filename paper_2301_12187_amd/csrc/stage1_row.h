// Stage 1, the walk of one wave over one source row k (Algorithm 1, Eq. 5a/5b
// of the paper), shared by the batched kernel and the single-launch path for
// small instances.
//
// Lanes own the targets l = lane + 64u.  The wave visits the sources
// m = k, k+1, ... in order and, for each, relaxes every l > m at once ("push"
// form of the algorithm's arg-min over the last block).  When the walk reaches
// m, every m' < m has been pushed, so lane(m)'s running minimum is the final
// Topt[k][m]; it is broadcast with a cross-lane read.  Sources are visited in
// ascending order and a candidate replaces the minimum only when strictly
// smaller, so the lowest arg-min m' is kept.  T[m][l] is read along l: coalesced.
#pragma once
#include "dpc_internal.h"

namespace dpc {

// The sources m of one 64-block, m in [mbeg, mend) with 64 ULO <= m < 64 (ULO + 1):
// only the registers u >= ULO still hold targets above m, and the finished
// value of source m sits in register ULO.
template <int S1_U, int S1_AHEAD, int ULO, bool T_IN_LDS>
__device__ __forceinline__ void stage1_block(int L, const int32_t* __restrict__ Tb, int k, int lane,
                                             int mbeg, int mend, int32_t (&cur)[S1_U],
                                             int32_t (&arg)[S1_U])
{
    const int ld = L + 1;
    // A lane's target l takes part in the step of source m when m < l <= L.  lt[u]
    // is l where l <= L and -1 beyond the row, so that "lt[u] > m" is the whole
    // test; lc[u] is l clamped into the row, so that every lane can load.
    int lt[S1_U], lc[S1_U];
#pragma unroll
    for (int u = ULO; u < S1_U; ++u) {
        const int l = lane + 64 * u;
        lt[u] = l <= L ? l : -1;
        lc[u] = min(l, L);
    }
    // The loads of T do not depend on the recurrence: fetch S1_AHEAD source rows
    // at once, then run their dependent steps from registers.  A target that
    // does not take part gets DPC_INF instead of T[m][l]: its candidate is then
    // at least DPC_INF and replaces nothing (the minimum starts at DPC_INF), so
    // the steps themselves need no test.
    for (int m0 = mbeg; m0 < mend; m0 += S1_AHEAD) {
        int32_t tv[S1_AHEAD][S1_U];
#pragma unroll
        for (int a = 0; a < S1_AHEAD; ++a) {
            const int m = min(m0 + a, mend - 1);
            const int32_t* Trow = Tb + (size_t)m * ld;
#pragma unroll
            for (int u = ULO; u < S1_U; ++u) {
                if constexpr (T_IN_LDS) {
                    // (every lane reads: cheaper there than a read under a lane mask)
                    const int32_t t = Trow[lc[u]];
                    tv[a][u] = lt[u] > m ? t : DPC_INF;
                } else {
                    // (only the lanes that take part load: half the traffic)
                    tv[a][u] = DPC_INF;
                    if (lt[u] > m) tv[a][u] = Trow[lc[u]];
                }
            }
        }
#pragma unroll
        for (int a = 0; a < S1_AHEAD; ++a) {
            const int m = m0 + a;
            if (m >= mend) break;
            // final Topt[k][m]: 0 for m == k, else the owner lane's minimum
            // (m is the same in every lane: a scalar lane read, not a permute)
            int32_t tm = __builtin_amdgcn_readlane(cur[ULO], m & 63);
            if (m == k) tm = 0;
#pragma unroll
            for (int u = ULO; u < S1_U; ++u) {
                // Both terms are <= DPC_INF = 2^30 - 1: the sum fits int32 and needs
                // no clamp to DPC_INF (a sum at or beyond it never replaces anything).
                const int32_t c = tm + tv[a][u];
                if (c < cur[u]) { cur[u] = c; arg[u] = m; }
            }
        }
    }
}

// S1_U: targets per lane (64 * S1_U > L); S1_AHEAD: source rows fetched per batch;
// T_IN_LDS: the table T of the instance has been copied to LDS.
// On return cur[u] = Topt[k][lane + 64u] and arg[u] = its arg-min for l > k.
// The walk goes through the 64-blocks of sources one after the other, each
// compiled for the registers it still needs.
template <int S1_U, int S1_AHEAD, bool T_IN_LDS>
__device__ __forceinline__ void stage1_row(int L, const int32_t* __restrict__ Tb, int k, int lane,
                                           int32_t (&cur)[S1_U], int32_t (&arg)[S1_U])
{
    static_assert(S1_U >= 1 && S1_U <= 4, "up to 256 targets");
#pragma unroll
    for (int u = 0; u < S1_U; ++u) { cur[u] = DPC_INF; arg[u] = k; }
    const int mlast = L;                                  // sources are m = k .. L-1
    if (k < 64) stage1_block<S1_U, S1_AHEAD, 0, T_IN_LDS>(L, Tb, k, lane, k, min(64, mlast), cur, arg);
    if constexpr (S1_U > 1)
        if (k < 128 && mlast > 64)
            stage1_block<S1_U, S1_AHEAD, 1, T_IN_LDS>(L, Tb, k, lane, max(k, 64), min(128, mlast), cur, arg);
    if constexpr (S1_U > 2)
        if (k < 192 && mlast > 128)
            stage1_block<S1_U, S1_AHEAD, 2, T_IN_LDS>(L, Tb, k, lane, max(k, 128), min(192, mlast), cur, arg);
    if constexpr (S1_U > 3)
        if (mlast > 192)
            stage1_block<S1_U, S1_AHEAD, 3, T_IN_LDS>(L, Tb, k, lane, max(k, 192), mlast, cur, arg);
}

}  // namespace dpc
