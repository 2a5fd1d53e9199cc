// Extended solver (Appendix B of the paper, "Extension on the Importance"):
// block importances I[k][l][a][b] that depend on whether the activations at the
// two ends of the block are kept (a at k, b at l).
//
//   ext_iopt_kernel      Algorithm 3: I_opt[k][l][a][b] = the best chain of
//                        blocks from k to l whose interior end points carry an
//                        identity activation (flag 0), as a max-plus interval
//                        DP, with the arg-max pointers of B_opt.
//   ext_expand_kernel    Algorithm 4 is Algorithm 2 on the states (l, a): they
//                        are laid out as a chain of 2L+3 virtual layers,
//                        v = 2l + a, plus one last layer that takes the better
//                        of (L, 0) and (L, 1); this kernel writes the virtual
//                        latency and importance tables, on which the ordinary
//                        stage-2 kernels then run unchanged.  Predecessors in
//                        ascending v are the (k', alpha') pairs in ascending
//                        order, so arg-max ties break as in the paper's loop.
//   ext_backtrack_kernel the set updates of Algorithm 4 (A, S, B) unrolled
//                        through the stored pointers.
#include "dpc_internal.h"

namespace dpc {

constexpr int X1_WAVES = 4;       // waves per workgroup

// One wave per (instance, k, a).  Lanes own the targets l = lane + 64u, both
// end flags b.  The running maximum starts from the single block (k, l) with
// flags (a, b); the wave then walks the split points m = k+1, k+2, ... in
// ascending order and pushes I_opt[k][m][a][0] + I[m][l][0][b] to every l > m.
// When the walk reaches m every smaller split point has been pushed, so the
// owner lane's maximum for b = 0 is the final I_opt[k][m][a][0]; it is
// broadcast with a lane read.  A candidate replaces the maximum only when
// strictly greater: the single block, then the lowest m, wins ties.
// The importances I[m][l][0][.] do not depend on the walk: X1_AHEAD rows of
// them are fetched at once (both flags b of a target are one 8-byte load).
// X1_U: targets per lane, 64 * X1_U > L.
// The walk of one wave for one (k, a).  PAIRS_IN_LDS: the pairs
// (I[m][l][0][0], I[m][l][0][1]) of the instance have been copied to LDS, sI[m * ld + l].
template <int X1_U, int X1_AHEAD, bool PAIRS_IN_LDS>
__device__ __forceinline__ void ext_iopt_row(int L, const float* __restrict__ Ib, const float2* sI,
                                             int k, int a, int lane, float (&best)[X1_U][2],
                                             int (&arg)[X1_U][2])
{
    const int ld = L + 1;
#pragma unroll
    for (int u = 0; u < X1_U; ++u) {
        const int l = lane + 64 * u;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            best[u][f] = (l > k && l <= L) ? Ib[i4_index(ld, k, l, a, f)] : -INFINITY;
            arg[u][f] = k;
        }
    }
    for (int m0 = k + 1; m0 < L; m0 += X1_AHEAD) {
        float2 iv[X1_AHEAD][X1_U];          // I[m][l][0][0], I[m][l][0][1]
#pragma unroll
        for (int x = 0; x < X1_AHEAD; ++x) {
            const int m = min(m0 + x, L - 1);
#pragma unroll
            for (int u = 0; u < X1_U; ++u) {
                const int l = lane + 64 * u;
                if constexpr (PAIRS_IN_LDS) {
                    // (every lane reads: cheaper there than a read under a lane mask)
                    const float2 v = sI[m * ld + min(l, L)];
                    iv[x][u] = (l > m && l <= L) ? v : make_float2(-INFINITY, -INFINITY);
                } else {
                    iv[x][u] = (l > m && l <= L) ? *(const float2*)(Ib + i4_index(ld, m, l, 0, 0))
                                                 : make_float2(-INFINITY, -INFINITY);
                }
            }
        }
#pragma unroll
        for (int x = 0; x < X1_AHEAD; ++x) {
            const int m = m0 + x;
            if (m >= L) break;
            float own = best[0][0];
            const int um = m >> 6;
#pragma unroll
            for (int u = 1; u < X1_U; ++u) own = (um == u) ? best[u][0] : own;
            const float vm = __builtin_bit_cast(
                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, own), m & 63));
#pragma unroll
            for (int u = 0; u < X1_U; ++u) {
                // (a target that does not take part got -inf at the load: its
                //  candidate is -inf and replaces nothing, so no test here)
                const float c0 = vm + iv[x][u].x;
                if (c0 > best[u][0]) { best[u][0] = c0; arg[u][0] = m; }
                const float c1 = vm + iv[x][u].y;
                if (c1 > best[u][1]) { best[u][1] = c1; arg[u][1] = m; }
            }
        }
    }
}

template <int X1_U>
__device__ __forceinline__ void ext_iopt_store(int L, size_t inst, int k, int a, int lane,
                                               const float (&best)[X1_U][2],
                                               const int (&arg)[X1_U][2], float* __restrict__ Iopt,
                                               uint8_t* __restrict__ bsplit)
{
    const int ld = L + 1;
#pragma unroll
    for (int u = 0; u < X1_U; ++u) {
        const int l = lane + 64 * u;
        if (l <= L) {
            const bool upper = l > k;
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                Iopt[inst + i4_index(ld, k, l, a, f)] = upper ? best[u][f] : 0.0f;
                bsplit[inst + i4_index(ld, k, l, a, f)] = upper ? (uint8_t)arg[u][f] : (uint8_t)0;
            }
        }
    }
}

template <int X1_U, int X1_AHEAD>
__global__ __launch_bounds__(64 * X1_WAVES) void ext_iopt_kernel(
    int L, const float* __restrict__ I4, float* __restrict__ Iopt, uint8_t* __restrict__ bsplit)
{
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * X1_WAVES + (threadIdx.x >> 6);   // = 2k + a
    const int k = w >> 1, a = w & 1;
    const int b = blockIdx.y;
    if (k > L) return;                      // whole wave leaves together
    const int ld = L + 1;
    const size_t inst = (size_t)b * ld * ld * 4;
    float best[X1_U][2];
    int arg[X1_U][2];
    ext_iopt_row<X1_U, X1_AHEAD, false>(L, I4 + inst, nullptr, k, a, lane, best, arg);
    ext_iopt_store<X1_U>(L, inst, k, a, lane, best, arg, Iopt, bsplit);
}

// Short chains in a batch: one workgroup per instance first copies the pairs
// I[m][l][0][.] that every walk reads into LDS (each of the 2 (L + 1) walks of an
// instance reads about half of them; from global memory that is the bandwidth
// of the second-level cache), then its waves take the (k, a) in turn.
constexpr int X1L_MAX_L = 63;

__global__ __launch_bounds__(1024) void ext_iopt_lds_kernel(
    int L, const float* __restrict__ I4, float* __restrict__ Iopt, uint8_t* __restrict__ bsplit)
{
    extern __shared__ float2 x1_pairs[];
    const int ld = L + 1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const size_t inst = (size_t)blockIdx.x * ld * ld * 4;
    const float* Ib = I4 + inst;
    for (int x = threadIdx.x; x < ld * ld; x += blockDim.x) {
        const int m = x / ld, l = x - m * ld;
        x1_pairs[x] = *(const float2*)(Ib + i4_index(ld, m, l, 0, 0));
    }
    __syncthreads();
    for (int w = wave; w < 2 * ld; w += nw) {
        const int k = w >> 1, a = w & 1;
        float best[1][2];
        int arg[1][2];
        ext_iopt_row<1, 8, true>(L, Ib, x1_pairs, k, a, lane, best, arg);
        ext_iopt_store<1>(L, inst, k, a, lane, best, arg, Iopt, bsplit);
    }
}

// Virtual tables of the chain of states: V = 2L+3 layers.  v = 2l + a for
// 0 <= l <= L; v = 2L+2 is the final layer.  An entry (u, v), u < v:
//   u = 0, v = 1          latency 0, importance +0  (D[0][t][1] = D[0][t][0] = +0)
//   same l, u != v        none
//   v <= 2L+1             latency Topt[k'][l], importance I_opt[k'][l][alpha'][a]
//   v = 2L+2              from (L, 0) and (L, 1): latency 0, importance +0
// "None" is latency DPC_INF (no budget reaches it) and importance -inf.
__global__ __launch_bounds__(256) void ext_expand_kernel(
    int L, const int32_t* __restrict__ Topt, const float* __restrict__ Iopt,
    int32_t* __restrict__ Tv, float* __restrict__ Iv)
{
    const int V = 2 * L + 3;
    const int b = blockIdx.y;
    const int x = blockIdx.x * 256 + threadIdx.x;
    if (x >= V * V) return;
    const int u = x / V, v = x - u * V;
    int32_t t;
    float imp;
    ToptRef{Topt, 1, L, Iopt}.operands(nullptr, b, V, u, v, t, imp);
    Tv[(size_t)b * V * V + x] = t;
    Iv[(size_t)b * V * V + x] = imp;
}

// One wave per query: from the final layer at budget T0 back to layer 0.
// Everything that steers the walk is wave-uniform.  Per DP step (k, alpha') ->
// (l, a) the wave reads one pointer byte, one latency, row k of `split` and the
// rows (k, ., alpha', 0/1) of `bsplit` (a byte, resp. a byte pair, per lane and
// 64 targets), then follows both pointer chains inside the block through lane
// reads.  Members come out from high to low into three lists in LDS and are
// written out ascending at the end; they strictly decrease along the walk
// (enforced), so no list holds more than L-1 entries whatever the tables hold.
constexpr int XB_WAVES = 4;       // queries per workgroup
constexpr int XB_U = 2;           // targets per lane: L <= DPC_EXT_MAX_L = 126

__global__ __launch_bounds__(64 * XB_WAVES) void ext_backtrack_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const uint8_t* __restrict__ split,
    const uint8_t* __restrict__ bsplit, const float* __restrict__ D,
    const uint8_t* __restrict__ Kx, int Q, const int32_t* __restrict__ q_inst,
    const int32_t* __restrict__ q_T0, int32_t* A, int32_t* __restrict__ A_len, int32_t* S,
    int32_t* __restrict__ S_len, int32_t* Bs, int32_t* __restrict__ B_len,
    float* __restrict__ obj, int32_t* __restrict__ lat, int32_t* __restrict__ a_last,
    int32_t* __restrict__ status)
{
    __shared__ int32_t listA[XB_WAVES][128];
    __shared__ int32_t listS[XB_WAVES][128];
    __shared__ int32_t listB[XB_WAVES][128];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = blockIdx.x * XB_WAVES + wv;
    if (q >= Q) return;                          // whole wave leaves together
    const int b = __builtin_amdgcn_readfirstlane(q_inst[q]);
    const int T0 = __builtin_amdgcn_readfirstlane(q_T0[q]);
    const int ld = L + 1, V = 2 * L + 3;
    int st = DPC_Q_OK;
    if (b < 0 || b >= B || T0 < 0 || T0 >= P) st = DPC_Q_BAD_QUERY;
    float top = -INFINITY;
    const float* Db = nullptr;
    const uint8_t* Kb = nullptr;
    if (st == DPC_Q_OK) {
        Db = D + (size_t)b * V * P;
        Kb = Kx + (size_t)b * V * P;
        top = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                                            __builtin_bit_cast(int, Db[(size_t)(V - 1) * P + T0])));
        if (top == -INFINITY) st = DPC_Q_INFEASIBLE;
    }
    if (st != DPC_Q_OK) {
        if (lane == 0) {
            A_len[q] = -1; S_len[q] = -1; B_len[q] = -1; obj[q] = -INFINITY; lat[q] = -1;
            a_last[q] = -1; status[q] = st;
        }
        return;
    }
    const int32_t* To = Topt + (size_t)b * ld * ld;
    const uint8_t* Sp = split + (size_t)b * ld * ld;
    const uint8_t* Bp = bsplit + (size_t)b * ld * ld * 4;
    int na = 0, ns = 0, nb = 0, total = 0;
    int v = __builtin_amdgcn_readfirstlane((int)Kb[(size_t)(V - 1) * P + T0]);   // (L, a_last)
    int l = v >> 1, a = v & 1, t = T0;
    const int alast = a;
    if (l != L) l = 0;                           // defensive: never true for stage-2 output
    while (l > 0) {
        const int u = __builtin_amdgcn_readfirstlane((int)Kb[(size_t)(2 * l + a) * P + t]);
        const int k = u >> 1, al = u & 1;
        if (k >= l) break;                       // defensive
        const int32_t w = __builtin_amdgcn_readfirstlane(To[k * ld + l]);
        // row k of split and rows (k, ., al, 0/1) of bsplit: target x in lane x & 63, register x >> 6
        int srow[XB_U], brow[XB_U];
#pragma unroll
        for (int uu = 0; uu < XB_U; ++uu) {
            const int x = lane + 64 * uu;
            srow[uu] = x <= L ? (int)Sp[k * ld + x] : 0;
            brow[uu] = x <= L ? (int)*(const uint16_t*)(Bp + i4_index(ld, k, x, al, 0)) : 0;
        }
        for (int x = l;;) {
            int src = srow[0];
#pragma unroll
            for (int uu = 1; uu < XB_U; ++uu) src = (x >> 6) == uu ? srow[uu] : src;
            const int m = __builtin_amdgcn_readlane(src, x & 63);
            if (m <= k || m >= x) break;         // m == k ends S_opt[k,l]; the rest is defensive
            if (lane == 0) listS[wv][ns] = m;
            ++ns;
            x = m;
        }
        for (int x = l, f = a;;) {
            int src = brow[0];
#pragma unroll
            for (int uu = 1; uu < XB_U; ++uu) src = (x >> 6) == uu ? brow[uu] : src;
            const int m = (__builtin_amdgcn_readlane(src, x & 63) >> (8 * f)) & 0xFF;
            if (m <= k || m >= x) break;
            if (lane == 0) listB[wv][nb] = m;
            ++nb;
            x = m;
            f = 0;
        }
        if (k > 0) {
            if (lane == 0) {
                if (al) listA[wv][na] = k;
                listS[wv][ns] = k;
                listB[wv][nb] = k;
            }
            na += al;
            ++ns;
            ++nb;
        }
        if (w > t) break;                        // defensive
        total += w; t -= w; l = k; a = al;
    }
    int32_t* Aq = A + (size_t)q * L;
    int32_t* Sq = S + (size_t)q * L;
    int32_t* Bq = Bs + (size_t)q * L;
    for (int x = lane; x < na; x += 64) Aq[x] = listA[wv][na - 1 - x];
    for (int x = lane; x < ns; x += 64) Sq[x] = listS[wv][ns - 1 - x];
    for (int x = lane; x < nb; x += 64) Bq[x] = listB[wv][nb - 1 - x];
    if (lane == 0) {
        A_len[q] = na; S_len[q] = ns; B_len[q] = nb; obj[q] = top; lat[q] = total;
        a_last[q] = alast; status[q] = DPC_Q_OK;
    }
}

hipError_t launch_ext_iopt(int B, int L, const float* I4, float* Iopt, uint8_t* bsplit, hipStream_t st)
{
    if (L <= X1L_MAX_L && B >= 128) {
        const int nt = 64 * std::min(16, 2 * (L + 1));
        const size_t lds = (size_t)(L + 1) * (L + 1) * sizeof(float2);
        hipLaunchKernelGGL(ext_iopt_lds_kernel, dim3(B), dim3(nt), lds, st, L, I4, Iopt, bsplit);
        return hipGetLastError();
    }
    dim3 grid((2 * (L + 1) + X1_WAVES - 1) / X1_WAVES, B);
    if (L < 64)
        hipLaunchKernelGGL((ext_iopt_kernel<1, 8>), grid, dim3(64 * X1_WAVES), 0, st, L, I4, Iopt, bsplit);
    else if (L < 128)
        hipLaunchKernelGGL((ext_iopt_kernel<2, 8>), grid, dim3(64 * X1_WAVES), 0, st, L, I4, Iopt, bsplit);
    else
        hipLaunchKernelGGL((ext_iopt_kernel<4, 4>), grid, dim3(64 * X1_WAVES), 0, st, L, I4, Iopt, bsplit);
    return hipGetLastError();
}

hipError_t launch_ext_expand(int B, int L, const int32_t* Topt, const float* Iopt, int32_t* Tv,
                             float* Iv, hipStream_t st)
{
    const int V = 2 * L + 3;
    dim3 grid((V * V + 255) / 256, B);
    hipLaunchKernelGGL(ext_expand_kernel, grid, dim3(256), 0, st, L, Topt, Iopt, Tv, Iv);
    return hipGetLastError();
}

hipError_t launch_ext_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                                const uint8_t* bsplit, const float* D, const uint8_t* Kx, int Q,
                                const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                                int32_t* A_len, int32_t* S, int32_t* S_len, int32_t* Bs,
                                int32_t* B_len, float* obj, int32_t* lat, int32_t* a_last,
                                int32_t* status, hipStream_t st)
{
    hipLaunchKernelGGL(ext_backtrack_kernel, dim3((Q + XB_WAVES - 1) / XB_WAVES),
                       dim3(64 * XB_WAVES), 0, st, B, L, P, Topt, split, bsplit, D, Kx, Q, q_inst,
                       q_T0, A, A_len, S, S_len, Bs, B_len, obj, lat, a_last, status);
    return hipGetLastError();
}

}  // namespace dpc
