// Set recovery: A[L,T0] and S[L,T0] of Algorithm 2 (set updates Eq. 7a/7b of
// the paper) rebuilt from the stored arg-max pointers K and, inside every
// block (i, j) of the chain, the arg-min pointers of Algorithm 1.
//
// One 64-lane wave per query; everything that steers the walk is
// wave-uniform.  Per block of the chain the wave reads one arg-max byte, one
// latency and the row i of `split` (L+1 bytes, one byte per lane and 64
// targets), and then follows the arg-min pointers inside the block through
// lane reads of that row instead of dependent loads.  Members come out from
// high to low into two lists in LDS and are written out in ascending order at
// the end.  Members strictly decrease along the walk (i < m < l <= j is
// enforced), so both sets hold at most L-1 entries whatever the tables
// contain.  Without stored pointers (K == NULL) the arg-max of a visited cell
// is found again as the lowest i whose candidate reproduces the stored cell
// bit for bit: the lanes test 64 predecessors at a time.
#include "dpc_internal.h"

namespace dpc {

constexpr int BT_WAVES = 4;        // queries per workgroup
constexpr int BT_U = 4;            // bytes of a split row per lane: L <= 255

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__global__ __launch_bounds__(64 * BT_WAVES) void backtrack_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const uint8_t* __restrict__ split,
    const float* __restrict__ I, const float* __restrict__ M, const uint8_t* __restrict__ K,
    int Q, const int32_t* __restrict__ q_inst, const int32_t* __restrict__ q_T0,
    int32_t* __restrict__ A, int32_t* __restrict__ A_len, int32_t* __restrict__ S,
    int32_t* __restrict__ S_len, float* __restrict__ obj, int32_t* __restrict__ lat,
    int32_t* __restrict__ status)
{
    __shared__ int32_t listA[BT_WAVES][256];
    __shared__ int32_t listS[BT_WAVES][256];
    const int lane = threadIdx.x & 63;
    const int wv = uniform(threadIdx.x >> 6);
    const int q = blockIdx.x * BT_WAVES + wv;
    if (q >= Q) return;                     // whole wave leaves together
    const int b = uniform(q_inst[q]);
    const int T0 = uniform(q_T0[q]);
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
        To = Topt + (size_t)b * ld * ld;
        Sp = split + (size_t)b * ld * ld;
        Ib = I + (size_t)b * ld * ld;
        Mb = M + (size_t)b * ld * P;
        Kb = K ? K + (size_t)b * ld * P : nullptr;
        top = __builtin_bit_cast(float, uniform(__builtin_bit_cast(int, Mb[(size_t)L * P + T0])));
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
            i = uniform((int)Kb[(size_t)j * P + t]);
        } else {
            // no stored pointer: the lowest i whose candidate equals the stored cell.
            // All predecessors are tested at once (j <= 255: four per lane), the
            // loads of a step issued together: latencies, then cells and importances.
            const float want = Mb[(size_t)j * P + t];
            int32_t wv[BT_U];
            float mv[BT_U], iv[BT_U];
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int ic = lane + 64 * u;
                wv[u] = ic < j ? To[ic * ld + j] : DPC_INF;
            }
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int ic = lane + 64 * u;
                const bool ok = ic < j && wv[u] <= t;
                mv[u] = ok ? Mb[(size_t)ic * P + (t - wv[u])] : -INFINITY;
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
        const int32_t w = uniform(To[i * ld + j]);
        // row i of split: byte l sits in lane l & 63, register l >> 6
        int row[BT_U];
#pragma unroll
        for (int u = 0; u < BT_U; ++u) {
            const int l = lane + 64 * u;
            row[u] = l <= L ? (int)Sp[i * ld + l] : 0;
        }
        int l = j;
        for (;;) {
            int src = row[0];
#pragma unroll
            for (int u = 1; u < BT_U; ++u) src = (l >> 6) == u ? row[u] : src;
            const int m = __builtin_amdgcn_readlane(src, l & 63);
            if (m <= i || m >= l) break;    // m == i ends S_opt[i,j]; the rest is defensive
            if (lane == 0) listS[wv][ns] = m;
            ++ns;
            l = m;
        }
        if (i > 0) {
            if (lane == 0) { listA[wv][na] = i; listS[wv][ns] = i; }
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
    for (int x = lane; x < na; x += 64) Aq[x] = listA[wv][na - 1 - x];
    for (int x = lane; x < ns; x += 64) Sq[x] = listS[wv][ns - 1 - x];
    if (lane == 0) {
        A_len[q] = na; S_len[q] = ns; obj[q] = top; lat[q] = total; status[q] = DPC_Q_OK;
    }
}

hipError_t launch_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                            const float* I, const float* M, const uint8_t* K, int Q,
                            const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                            int32_t* A_len, int32_t* S, int32_t* S_len, float* obj,
                            int32_t* lat, int32_t* status, hipStream_t st)
{
    dim3 grid((Q + BT_WAVES - 1) / BT_WAVES);
    hipLaunchKernelGGL(backtrack_kernel, grid, dim3(64 * BT_WAVES), 0, st, B, L, P, Topt, split, I,
                       M, K, Q, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status);
    return hipGetLastError();
}

}  // namespace dpc
