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
template <int S1_U, int S1_AHEAD, int ULO>
__device__ __forceinline__ void stage1_block(int L, const int32_t* __restrict__ Tb, int k, int lane,
                                             int mbeg, int mend, int32_t (&cur)[S1_U],
                                             int32_t (&arg)[S1_U])
{
    const int ld = L + 1;
    // The loads of T do not depend on the recurrence: fetch S1_AHEAD source rows
    // at once, then run their dependent steps from registers.
    for (int m0 = mbeg; m0 < mend; m0 += S1_AHEAD) {
        int32_t tv[S1_AHEAD][S1_U];
#pragma unroll
        for (int a = 0; a < S1_AHEAD; ++a) {
            const int m = min(m0 + a, mend - 1);
            const int32_t* Trow = Tb + (size_t)m * ld;
#pragma unroll
            for (int u = ULO; u < S1_U; ++u) {
                const int l = lane + 64 * u;
                tv[a][u] = (l > m && l <= L) ? Trow[l] : DPC_INF;
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
                const int l = lane + 64 * u;
                if (l > m && l <= L) {
                    // Both terms are <= DPC_INF = 2^30 - 1: the sum fits int32.  It
                    // needs no clamp to DPC_INF: the minimum starts there, so a sum
                    // at or beyond it never replaces anything.
                    const int32_t c = tm + tv[a][u];
                    if (c < cur[u]) { cur[u] = c; arg[u] = m; }
                }
            }
        }
    }
}

// S1_U: targets per lane (64 * S1_U > L); S1_AHEAD: source rows fetched per batch.
// On return cur[u] = Topt[k][lane + 64u] and arg[u] = its arg-min for l > k.
// The walk goes through the 64-blocks of sources one after the other, each
// compiled for the registers it still needs.
template <int S1_U, int S1_AHEAD>
__device__ __forceinline__ void stage1_row(int L, const int32_t* __restrict__ Tb, int k, int lane,
                                           int32_t (&cur)[S1_U], int32_t (&arg)[S1_U])
{
    static_assert(S1_U >= 1 && S1_U <= 4, "up to 256 targets");
#pragma unroll
    for (int u = 0; u < S1_U; ++u) { cur[u] = DPC_INF; arg[u] = k; }
    const int mlast = L;                                  // sources are m = k .. L-1
    if (k < 64) stage1_block<S1_U, S1_AHEAD, 0>(L, Tb, k, lane, k, min(64, mlast), cur, arg);
    if constexpr (S1_U > 1)
        if (k < 128 && mlast > 64)
            stage1_block<S1_U, S1_AHEAD, 1>(L, Tb, k, lane, max(k, 64), min(128, mlast), cur, arg);
    if constexpr (S1_U > 2)
        if (k < 192 && mlast > 128)
            stage1_block<S1_U, S1_AHEAD, 2>(L, Tb, k, lane, max(k, 128), min(192, mlast), cur, arg);
    if constexpr (S1_U > 3)
        if (mlast > 192)
            stage1_block<S1_U, S1_AHEAD, 3>(L, Tb, k, lane, max(k, 192), mlast, cur, arg);
}

}  // namespace dpc
