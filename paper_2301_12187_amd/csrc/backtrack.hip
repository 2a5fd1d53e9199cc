// Set recovery: A[L,T0] and S[L,T0] of Algorithm 2 (set updates Eq. 7a/7b of
// the paper) rebuilt from the stored arg-max pointers K and, inside every
// block (i, j) of the chain, the arg-min pointers of Algorithm 1.  One lane per
// query; at most L pointer steps plus at most L split steps, all integer.
// The walk visits indices from high to low; the members are written in that
// order and each list is then reversed in place.  Members strictly decrease
// along the walk (i < m < l <= j is enforced), so both sets hold at most L-1
// entries whatever the tables contain.
#include "dpc_internal.h"

namespace dpc {

__device__ __forceinline__ int argmax_of_cell(int L, int P, const int32_t* To, const float* Ib,
                                              const float* Mb, const uint8_t* Kb, int j, int t)
{
    if (Kb) return Kb[(size_t)j * P + t];
    // no stored pointer: the lowest i whose candidate equals the stored cell
    const int ld = L + 1;
    const float want = Mb[(size_t)j * P + t];
    for (int i = 0; i < j; ++i) {
        const int32_t w = To[i * ld + j];
        if (w <= t) {
            const float c = Mb[(size_t)i * P + (t - w)] + Ib[i * ld + j];
            if (c == want) return i;
        }
    }
    return DPC_NOARG;   // unreachable for a table produced by stage 2
}

__global__ __launch_bounds__(64) void backtrack_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const uint8_t* __restrict__ split,
    const float* __restrict__ I, const float* __restrict__ M, const uint8_t* __restrict__ K,
    int Q, const int32_t* __restrict__ q_inst, const int32_t* __restrict__ q_T0,
    int32_t* A, int32_t* __restrict__ A_len, int32_t* S,
    int32_t* __restrict__ S_len, float* __restrict__ obj, int32_t* __restrict__ lat,
    int32_t* __restrict__ status)
{
    const int q = blockIdx.x * 64 + threadIdx.x;
    if (q >= Q) return;
    const int b = q_inst[q];
    const int T0 = q_T0[q];
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
        top = Mb[(size_t)L * P + T0];
        if (top == -INFINITY) st = DPC_Q_INFEASIBLE;
    }
    if (st != DPC_Q_OK) {
        A_len[q] = -1; S_len[q] = -1; obj[q] = -INFINITY; lat[q] = -1; status[q] = st;
        return;
    }
    // one walk: members come out from high to low and are written in that order,
    // then each list is reversed in place by the same lane
    int na = 0, ns = 0, total = 0;
    int32_t* Aq = A + (size_t)q * L;
    int32_t* Sq = S + (size_t)q * L;
    {
        int j = L, t = T0;
        while (j > 0) {
            const int i = argmax_of_cell(L, P, To, Ib, Mb, Kb, j, t);
            if (i >= j) break;              // defensive: never true for stage-2 output
            int l = j;
            for (;;) {
                const int m = Sp[i * ld + l];
                if (m <= i || m >= l) break;   // m == i ends S_opt[i,j]; the rest is defensive
                Sq[ns++] = m;
                l = m;
            }
            if (i > 0) {
                Aq[na++] = i;
                Sq[ns++] = i;
            }
            const int32_t w = To[i * ld + j];
            if (w > t) break;               // defensive: never true for stage-2 output
            total += w; t -= w; j = i;
        }
    }
    for (int a = 0, b2 = na - 1; a < b2; ++a, --b2) {
        const int32_t x = Aq[a]; Aq[a] = Aq[b2]; Aq[b2] = x;
    }
    for (int a = 0, b2 = ns - 1; a < b2; ++a, --b2) {
        const int32_t x = Sq[a]; Sq[a] = Sq[b2]; Sq[b2] = x;
    }
    A_len[q] = na; S_len[q] = ns; obj[q] = top; lat[q] = total; status[q] = DPC_Q_OK;
}

hipError_t launch_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                            const float* I, const float* M, const uint8_t* K, int Q,
                            const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                            int32_t* A_len, int32_t* S, int32_t* S_len, float* obj,
                            int32_t* lat, int32_t* status, hipStream_t st)
{
    dim3 grid((Q + 63) / 64);
    hipLaunchKernelGGL(backtrack_kernel, grid, dim3(64), 0, st, B, L, P, Topt, split, I, M, K, Q,
                       q_inst, q_T0, A, A_len, S, S_len, obj, lat, status);
    return hipGetLastError();
}

}  // namespace dpc
