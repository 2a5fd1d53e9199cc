// Set recovery, batched: one 64-lane wave per query (the walk itself is in
// backtrack_walk.h).
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

hipError_t launch_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                            const float* I, const float* M, const uint8_t* K, int Q,
                            const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                            int32_t* A_len, int32_t* S, int32_t* S_len, float* obj,
                            int32_t* lat, int32_t* status, int share, hipStream_t st)
{
    dim3 grid((Q + BT_WAVES - 1) / BT_WAVES);
    hipLaunchKernelGGL(backtrack_kernel, grid, dim3(64 * BT_WAVES), 0, st, B, L, P, Topt, split, I,
                       M, K, Q, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status, share);
    return hipGetLastError();
}

}  // namespace dpc
