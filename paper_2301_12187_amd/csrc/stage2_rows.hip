// Stage 2, row-at-a-time family: one launch per row j of Algorithm 2
// (recurrence Eq. 7 of the paper).  One lane per (instance, budget t); the
// lane walks the predecessors i = 0 .. j-1 in ascending order and keeps a
// candidate only when strictly greater, which yields the lowest arg-max.
// Topt[i][j] and I[i][j] are wave-uniform (scalar loads); M[i][t - Topt[i][j]]
// is a shifted, contiguous window of row i: coalesced.  Every row comes from
// global memory, so this family is bound by L2 / HBM reads; it serves tables
// narrower than 16 budgets, which the persistent family does not take, and as
// a plain cross-check of it in the tests.
#include "dpc_internal.h"

namespace dpc {

constexpr int S2R_THREADS = 256;

__global__ __launch_bounds__(S2R_THREADS) void stage2_row_kernel(
    int L, int P, int j, ToptRef Topt, const float* __restrict__ I,
    float* M, uint8_t* K)
{
    const int t = blockIdx.x * S2R_THREADS + threadIdx.x;
    const int b = blockIdx.y;
    if (t >= P) return;
    const int ld = L + 1;
    const int32_t* To = Topt.of(b, ld);
    const float* Ib = I + (size_t)b * ld * ld;
    float* Mb = M + (size_t)b * ld * P;

    float best = (j == 0) ? 0.0f : -INFINITY;
    int arg = DPC_NOARG;
    for (int i = 0; i < j; ++i) {
        const int32_t w = To[i * ld + j];
        const float imp = Ib[i * ld + j];
        if (w <= t) {
            const float c = Mb[(size_t)i * P + (t - w)] + imp;
            if (c > best) { best = c; arg = i; }
        }
    }
    Mb[(size_t)j * P + t] = best;
    if (K) K[((size_t)b * ld + j) * P + t] = (uint8_t)arg;
}

hipError_t launch_stage2_rows(int B, int L, int P, ToptRef Topt, const float* I,
                              float* M, uint8_t* K, hipStream_t st)
{
    dim3 grid((P + S2R_THREADS - 1) / S2R_THREADS, B);
    for (int j = 0; j <= L; ++j) {
        hipLaunchKernelGGL(stage2_row_kernel, grid, dim3(S2R_THREADS), 0, st, L, P, j, Topt, I,
                           M, K);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace dpc
