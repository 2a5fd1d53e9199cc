// Stage 1: min-plus interval DP over merged-block latencies (Algorithm 1,
// Eq. 5a/5b of the paper).
//
// Row k of Topt depends only on row k and on T, so every (instance, k) pair is
// an independent single-source shortest-path problem on the DAG m -> l with
// weight T[m][l].  One 64-lane wave owns one (instance, k); its walk is in
// stage1_row.h.
#include "stage1_row.h"

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
    stage1_row<S1_U, S1_AHEAD, false>(L, Tb, k, lane, cur, arg);
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

// Short chains: one workgroup per instance first copies the whole table T into
// LDS (coalesced), then its waves take the source rows k = wave, wave + NW, ...
// and walk them from there.  The walk is a chain of dependent steps; what it
// waited for in the kernel above was the latency of its row fetches.
constexpr int S1L_MAX_L = 63;     // measured: faster up to here (0.044 vs 0.056 ms at L = 53, B = 1024), slower at L = 100

template <int S1_U>
__global__ __launch_bounds__(1024) void stage1_lds_kernel(
    int L, const int32_t* __restrict__ T, int32_t* __restrict__ Topt, uint8_t* __restrict__ split)
{
    extern __shared__ int32_t s1_T[];
    const int ld = L + 1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const size_t inst = (size_t)blockIdx.x * ld * ld;
    for (int x = threadIdx.x; x < ld * ld; x += blockDim.x) s1_T[x] = T[inst + x];
    __syncthreads();
    for (int k = wave; k <= L; k += nw) {
        int32_t cur[S1_U];
        int32_t arg[S1_U];
        stage1_row<S1_U, 8, true>(L, s1_T, k, lane, cur, arg);
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
}

hipError_t launch_stage1(int B, int L, const int32_t* T, int32_t* Topt, uint8_t* split,
                         hipStream_t st)
{
    // (a few instances are better off spread over many workgroups, one wave per row)
    if (L <= S1L_MAX_L && B >= 128) {
        const int nt = 64 * std::min(16, L + 1);
        const size_t lds = (size_t)(L + 1) * (L + 1) * sizeof(int32_t);
        hipLaunchKernelGGL((stage1_lds_kernel<1>), dim3(B), dim3(nt), lds, st, L, T, Topt, split);
        return hipGetLastError();
    }
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
