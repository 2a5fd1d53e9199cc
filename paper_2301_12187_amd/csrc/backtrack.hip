// Set recovery, batched: one 64-lane wave per query (the walk itself is in
// backtrack_walk.h), or sixteen lanes per query for long lists over short chains.
#include "backtrack_walk.h"

namespace dpc {

constexpr int BT_WAVES = 4;        // queries per workgroup

__global__ __launch_bounds__(64 * BT_WAVES) void backtrack_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const uint8_t* __restrict__ split,
    const float* __restrict__ I, const float* __restrict__ M, const uint8_t* __restrict__ K,
    int Q, const int32_t* __restrict__ q_inst, const int32_t* __restrict__ q_T0,
    int32_t* __restrict__ A, int32_t* __restrict__ A_len, int32_t* __restrict__ S,
    int32_t* __restrict__ S_len, float* __restrict__ obj, int32_t* __restrict__ lat,
    int32_t* __restrict__ status, int share)
{
    __shared__ int32_t listA[BT_WAVES][256];
    __shared__ int32_t listS[BT_WAVES][256];
    const int lane = threadIdx.x & 63;
    const int wv = bt_uniform(threadIdx.x >> 6);
    const int q = blockIdx.x * BT_WAVES + wv;
    if (q >= Q) return;                     // whole wave leaves together
    const int b = bt_uniform(q_inst[q]);
    const int T0 = bt_uniform(q_T0[q]);
    backtrack_query<false>(q, b, T0, B, L, P, Topt, split, I, M, K, A, A_len, S, S_len, obj, lat,
                           status, listA[wv], listS[wv], lane, share);
}

// The same walk for long query lists over short chains (L <= 63, stored
// pointers): four queries per wave, sixteen lanes each.  One wave per query is
// bound by its chain of dependent loads, not by instructions, so the time of a
// long list is the number of rounds of resident waves times that latency;
// four queries per wave cut the rounds by four.  What is wave-uniform above is
// uniform within a group of sixteen lanes here; groups that finish early wait
// for the slowest of their wave.  Byte l of row i of `split` sits in lane
// l & 15, register l >> 4 of its group.
constexpr int BTQ_GROUP = 16;      // lanes per query
constexpr int BTQ_PER_WG = 64 * BT_WAVES / BTQ_GROUP;
constexpr int BTQ_MAX_L = 63;
constexpr int BTQ_U = (BTQ_MAX_L + 1) / BTQ_GROUP;   // bytes of a split row per lane

__global__ __launch_bounds__(64 * BT_WAVES) void backtrack_quarter_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const uint8_t* __restrict__ split,
    const float* __restrict__ M, const uint8_t* __restrict__ K, int Q,
    const int32_t* __restrict__ q_inst, const int32_t* __restrict__ q_T0, int32_t* __restrict__ A,
    int32_t* __restrict__ A_len, int32_t* __restrict__ S, int32_t* __restrict__ S_len,
    float* __restrict__ obj, int32_t* __restrict__ lat, int32_t* __restrict__ status, int share)
{
    __shared__ int32_t lists[BTQ_PER_WG][2][BTQ_MAX_L + 1];
    const int slot = threadIdx.x / BTQ_GROUP;
    const int gl = threadIdx.x & (BTQ_GROUP - 1);
    const int q = blockIdx.x * BTQ_PER_WG + slot;
    int32_t* const listA = lists[slot][0];
    int32_t* const listS = lists[slot][1];
    const int ld = L + 1;
    int st = DPC_Q_OK, b = 0, T0 = 0;
    if (q < Q) {
        b = q_inst[q];
        T0 = q_T0[q];
        if (b < 0 || b >= B || T0 < 0 || T0 >= P) st = DPC_Q_BAD_QUERY;
    }
    const bool live = q < Q;
    const bool valid = live && st == DPC_Q_OK;
    const size_t tb = valid ? (size_t)(share > 1 ? b / share : b) : 0;
    const size_t bb = valid ? (size_t)b : 0;
    const int32_t* To = Topt + tb * ld * ld;
    const uint8_t* Sp = split + tb * ld * ld;
    const float* Mb = M + bb * ld * P;
    const uint8_t* Kb = K + bb * ld * P;
    float top = -INFINITY;
    if (valid) {
        top = Mb[(size_t)L * P + T0];
        if (top == -INFINITY) st = DPC_Q_INFEASIBLE;
    }
    int na = 0, ns = 0, total = 0;
    int j = (valid && st == DPC_Q_OK) ? L : 0, t = T0;
    while (j > 0) {
        const int i = (int)Kb[(size_t)j * P + t];
        if (i >= j) break;                  // defensive: never true for stage-2 output
        const int32_t w = To[i * ld + j];
        int row[BTQ_U];
#pragma unroll
        for (int u = 0; u < BTQ_U; ++u) {
            const int l = gl + BTQ_GROUP * u;
            row[u] = l <= L ? (int)Sp[i * ld + l] : 0;
        }
        int l = j;
        for (;;) {
            int src = row[0];
#pragma unroll
            for (int u = 1; u < BTQ_U; ++u) src = (l >> 4) == u ? row[u] : src;
            const int m = __shfl(src, l & (BTQ_GROUP - 1), BTQ_GROUP);
            if (m <= i || m >= l) break;    // m == i ends S_opt[i,j]; the rest is defensive
            if (gl == 0) listS[ns] = m;
            ++ns;
            l = m;
        }
        if (i > 0) {
            if (gl == 0) { listA[na] = i; listS[ns] = i; }
            ++na;
            ++ns;
        }
        if (w > t) break;                   // defensive: never true for stage-2 output
        total += w; t -= w; j = i;
    }
    if (!live) return;
    if (st != DPC_Q_OK) {
        if (gl == 0) {
            A_len[q] = -1; S_len[q] = -1; obj[q] = -INFINITY; lat[q] = -1; status[q] = st;
        }
        return;
    }
    // (the lanes of the group read what its lane 0 wrote: same wave, in order)
    int32_t* Aq = A + (size_t)q * L;
    int32_t* Sq = S + (size_t)q * L;
    for (int x = gl; x < na; x += BTQ_GROUP) Aq[x] = listA[na - 1 - x];
    for (int x = gl; x < ns; x += BTQ_GROUP) Sq[x] = listS[ns - 1 - x];
    if (gl == 0) {
        A_len[q] = na; S_len[q] = ns; obj[q] = top; lat[q] = total; status[q] = DPC_Q_OK;
    }
}

hipError_t launch_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                            const float* I, const float* M, const uint8_t* K, int Q,
                            const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                            int32_t* A_len, int32_t* S, int32_t* S_len, float* obj,
                            int32_t* lat, int32_t* status, int share, hipStream_t st)
{
    // (enough queries for several rounds of resident waves: four to a wave)
    if (K != nullptr && L <= BTQ_MAX_L && Q >= 16384) {
        dim3 gridq((Q + BTQ_PER_WG - 1) / BTQ_PER_WG);
        hipLaunchKernelGGL(backtrack_quarter_kernel, gridq, dim3(64 * BT_WAVES), 0, st, B, L, P, Topt,
                           split, M, K, Q, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status, share);
        return hipGetLastError();
    }
    dim3 grid((Q + BT_WAVES - 1) / BT_WAVES);
    hipLaunchKernelGGL(backtrack_kernel, grid, dim3(64 * BT_WAVES), 0, st, B, L, P, Topt, split, I,
                       M, K, Q, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status, share);
    return hipGetLastError();
}

}  // namespace dpc
