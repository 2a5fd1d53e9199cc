// Set recovery for one query by one 64-lane wave: the walk shared by the
// batched kernel (backtrack.hip) and the single-launch path for small instances
// (fused_small.hip).  A[L,T0] and S[L,T0] of Algorithm 2 (set updates Eq. 7a/7b
// of the paper) are rebuilt from the stored arg-max pointers K and, inside
// every block (i, j) of the chain, the arg-min pointers of Algorithm 1.
//
// Everything that steers the walk is wave-uniform.  Per block of the chain the
// wave reads one arg-max byte, one latency and the row i of `split` (L+1
// bytes, one byte per lane and 64 targets), and then follows the arg-min
// pointers inside the block through lane reads of that row instead of
// dependent loads.  Members come out from high to low into two lists in LDS
// and are written out in ascending order at the end.  Members strictly
// decrease along the walk (i < m < l <= j is enforced), so both sets hold at
// most L-1 entries whatever the tables contain.  Without stored pointers
// (K == NULL) the arg-max of a visited cell is found again as the lowest i
// whose candidate reproduces the stored cell bit for bit: the lanes test 64
// predecessors at a time.
#pragma once
#include "dpc_internal.h"

namespace dpc {

constexpr int BT_U = 4;            // bytes of a split row per lane: L <= 255

__device__ __forceinline__ int bt_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Loads of the tables the walk reads.  AGENT: the tables were written earlier
// in the same launch (by this workgroup), so they are read at agent scope,
// past any line the compute unit's vector cache may hold from before.
template <bool AGENT, class T>
__device__ __forceinline__ T bt_ld(const T* p)
{
    if constexpr (AGENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}

// One query (instance b, budget T0), answered into entry q of the outputs.
// listA / listS: this wave's two lists in LDS, room for L entries each.
template <bool AGENT>
__device__ __forceinline__ void backtrack_query(
    int q, int b, int T0, int B, int L, int P, const int32_t* __restrict__ Topt,
    const uint8_t* __restrict__ split, const float* __restrict__ I, const float* M,
    const uint8_t* K, int32_t* __restrict__ A, int32_t* __restrict__ A_len,
    int32_t* __restrict__ S, int32_t* __restrict__ S_len, float* __restrict__ obj,
    int32_t* __restrict__ lat, int32_t* __restrict__ status, int32_t* listA, int32_t* listS, int lane,
    int share = 1)
{
    int st = DPC_Q_OK;
    if (b < 0 || b >= B || T0 < 0 || T0 >= P) st = DPC_Q_BAD_QUERY;
    const int ld = L + 1;
    const int32_t* To = nullptr;
    const uint8_t* Sp = nullptr;
    const float* Ib = nullptr;
    const float* Mb = nullptr;
    const uint8_t* Kb = nullptr;
    float top = -INFINITY;
    if (st == DPC_Q_OK) {
        // (share > 1: instance b uses the stage-1 tables of network b / share)
        const size_t tb = (size_t)(share > 1 ? b / share : b);
        To = Topt + tb * ld * ld;
        Sp = split + tb * ld * ld;
        Ib = I + (size_t)b * ld * ld;
        Mb = M + (size_t)b * ld * P;
        Kb = K ? K + (size_t)b * ld * P : nullptr;
        top = __builtin_bit_cast(float, bt_uniform(__builtin_bit_cast(int, bt_ld<AGENT>(&Mb[(size_t)L * P + T0]))));
        if (top == -INFINITY) st = DPC_Q_INFEASIBLE;
    }
    if (st != DPC_Q_OK) {
        if (lane == 0) {
            A_len[q] = -1; S_len[q] = -1; obj[q] = -INFINITY; lat[q] = -1; status[q] = st;
        }
        return;
    }
    int na = 0, ns = 0, total = 0;
    int j = L, t = T0;
    while (j > 0) {
        int i;
        if (Kb) {
            i = bt_uniform((int)bt_ld<AGENT>(&Kb[(size_t)j * P + t]));
        } else {
            // no stored pointer: the lowest i whose candidate equals the stored cell.
            // All predecessors are tested at once (j <= 255: four per lane), the
            // loads of a step issued together: latencies, then cells and importances.
            const float want = bt_ld<AGENT>(&Mb[(size_t)j * P + t]);
            int32_t wv[BT_U];
            float mv[BT_U], iv[BT_U];
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int ic = lane + 64 * u;
                wv[u] = ic < j ? bt_ld<AGENT>(&To[ic * ld + j]) : DPC_INF;
            }
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int ic = lane + 64 * u;
                const bool ok = ic < j && wv[u] <= t;
                mv[u] = ok ? bt_ld<AGENT>(&Mb[(size_t)ic * P + (t - wv[u])]) : -INFINITY;
                iv[u] = ok ? Ib[ic * ld + j] : -INFINITY;
            }
            i = DPC_NOARG;                  // unreachable for a table produced by stage 2
#pragma unroll
            for (int u = BT_U - 1; u >= 0; --u) {
                const bool hit = lane + 64 * u < j && wv[u] <= t && mv[u] + iv[u] == want;
                const unsigned long long mask = __ballot(hit);
                if (mask != 0) i = 64 * u + __builtin_ctzll(mask);
            }
        }
        if (i >= j) break;                  // defensive: never true for stage-2 output
        const int32_t w = bt_uniform(bt_ld<AGENT>(&To[i * ld + j]));
        // row i of split: byte l sits in lane l & 63, register l >> 6
        int row[BT_U];
#pragma unroll
        for (int u = 0; u < BT_U; ++u) {
            const int l = lane + 64 * u;
            row[u] = l <= L ? (int)bt_ld<AGENT>(&Sp[i * ld + l]) : 0;
        }
        int l = j;
        for (;;) {
            int src = row[0];
#pragma unroll
            for (int u = 1; u < BT_U; ++u) src = (l >> 6) == u ? row[u] : src;
            const int m = __builtin_amdgcn_readlane(src, l & 63);
            if (m <= i || m >= l) break;    // m == i ends S_opt[i,j]; the rest is defensive
            if (lane == 0) listS[ns] = m;
            ++ns;
            l = m;
        }
        if (i > 0) {
            if (lane == 0) { listA[na] = i; listS[ns] = i; }
            ++na;
            ++ns;
        }
        if (w > t) break;                   // defensive: never true for stage-2 output
        total += w; t -= w; j = i;
    }
    // the lists were filled from high to low: write them out ascending
    // (same wave wrote and reads the LDS lists: no barrier needed beyond its own order)
    int32_t* Aq = A + (size_t)q * L;
    int32_t* Sq = S + (size_t)q * L;
    for (int x = lane; x < na; x += 64) Aq[x] = listA[na - 1 - x];
    for (int x = lane; x < ns; x += 64) Sq[x] = listS[ns - 1 - x];
    if (lane == 0) {
        A_len[q] = na; S_len[q] = ns; obj[q] = top; lat[q] = total; status[q] = DPC_Q_OK;
    }
}

}  // namespace dpc
