// Stage 1: min-plus interval DP over merged-block latencies (Algorithm 1,
// Eq. 5a/5b of the paper).
//
// Row k of Topt depends only on row k and on T, so every (instance, k) pair is
// an independent single-source shortest-path problem on the DAG m -> l with
// weight T[m][l].  One 64-lane wave owns one (instance, k).  Lanes own the
// targets l = lane + 64u; the wave walks the sources m = k, k+1, ... in order
// and, for each, relaxes every l > m at once ("push" form of the algorithm's
// arg-min over the last block).  When the walk reaches m, every m' < m has been
// pushed, so lane(m)'s running minimum is the final Topt[k][m]; it is broadcast
// with a cross-lane read.  Sources are visited in ascending order and a
// candidate replaces the minimum only when strictly smaller, so the lowest
// arg-min m' is kept.  T[m][l] is read along l: coalesced.
#include "dpc_internal.h"

namespace dpc {

constexpr int S1_WAVES = 4;       // waves per workgroup

// S1_U: targets per lane (64 * S1_U > L); S1_AHEAD: source rows fetched per batch
template <int S1_U, int S1_AHEAD>
__global__ __launch_bounds__(64 * S1_WAVES) void stage1_kernel(
    int L, const int32_t* __restrict__ T, int32_t* __restrict__ Topt,
    uint8_t* __restrict__ split)
{
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * S1_WAVES + (threadIdx.x >> 6);
    const int b = blockIdx.y;
    if (k > L) return;                      // whole wave leaves together
    const int ld = L + 1;
    const size_t inst = (size_t)b * ld * ld;
    const int32_t* Tb = T + inst;

    int32_t cur[S1_U];
    int32_t arg[S1_U];
#pragma unroll
    for (int u = 0; u < S1_U; ++u) { cur[u] = DPC_INF; arg[u] = k; }

    // The loads of T do not depend on the recurrence: fetch S1_AHEAD source rows
    // at once, then run their dependent steps from registers.
    for (int m0 = k; m0 < L; m0 += S1_AHEAD) {
        int32_t tv[S1_AHEAD][S1_U];
#pragma unroll
        for (int a = 0; a < S1_AHEAD; ++a) {
            const int m = min(m0 + a, L - 1);
            const int32_t* Trow = Tb + (size_t)m * ld;
#pragma unroll
            for (int u = 0; u < S1_U; ++u) {
                const int l = lane + 64 * u;
                tv[a][u] = (l > m && l <= L) ? Trow[l] : DPC_INF;
            }
        }
#pragma unroll
        for (int a = 0; a < S1_AHEAD; ++a) {
            const int m = m0 + a;
            if (m >= L) break;
            // final Topt[k][m]: 0 for m == k, else the owner lane's minimum
            int32_t own = cur[0];
            const int um = m >> 6;
#pragma unroll
            for (int u = 1; u < S1_U; ++u) own = (um == u) ? cur[u] : own;
            int32_t tm = __shfl(own, m & 63, 64);
            if (m == k) tm = 0;
#pragma unroll
            for (int u = 0; u < S1_U; ++u) {
                const int l = lane + 64 * u;
                if (l > m && l <= L) {
                    // both terms are <= DPC_INF = 2^30 - 1: the sum fits int32
                    int32_t c = tm + tv[a][u];
                    c = c > DPC_INF ? DPC_INF : c;
                    if (c < cur[u]) { cur[u] = c; arg[u] = m; }
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < S1_U; ++u) {
        const int l = lane + 64 * u;
        if (l <= L) {
            const bool upper = l > k;
            Topt[inst + (size_t)k * ld + l] = upper ? cur[u] : 0;
            split[inst + (size_t)k * ld + l] = upper ? (uint8_t)arg[u] : (uint8_t)0;
        }
    }
}

hipError_t launch_stage1(int B, int L, const int32_t* T, int32_t* Topt, uint8_t* split,
                         hipStream_t st)
{
    dim3 grid((L + 1 + S1_WAVES - 1) / S1_WAVES, B);
    // short chains keep one or two targets per lane: fewer instructions per
    // step and room to fetch more source rows at once
    if (L < 64)
        hipLaunchKernelGGL((stage1_kernel<1, 16>), grid, dim3(64 * S1_WAVES), 0, st, L, T, Topt, split);
    else if (L < 128)
        hipLaunchKernelGGL((stage1_kernel<2, 8>), grid, dim3(64 * S1_WAVES), 0, st, L, T, Topt, split);
    else
        hipLaunchKernelGGL((stage1_kernel<4, 8>), grid, dim3(64 * S1_WAVES), 0, st, L, T, Topt, split);
    return hipGetLastError();
}

}  // namespace dpc
