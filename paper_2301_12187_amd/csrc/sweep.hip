// Steps around the solver in a sweep over hyper-parameters: the importance
// normalisation (appendix "Evaluating and Normalizing the Importance" of the
// paper), the trade-off curve read off the last row of Algorithm 2's table,
// and the latency of a network merged at a given ordered set (the constraint
// side of Eq. 4; with A in place of S, the ablation on the set to be merged).
// All three are small, memory-bound passes.
#include "dpc_internal.h"

namespace dpc {

// ---- importance normalisation ------------------------------------------------
// One workgroup per (instance, alpha).  The size-one entries (at most 255 x 4)
// go to LDS, one thread adds them up in ascending order in binary64 (the order
// fixes the rounding), and every thread then shifts its share of the table.
constexpr int SH_NT = 256;

__global__ __launch_bounds__(SH_NT) void importance_shift_kernel(
    int L, int F, int n_alpha, const float* __restrict__ I_raw, const float* __restrict__ alpha,
    float* __restrict__ I_out, double* __restrict__ mean_out)
{
    __shared__ float d[DPC_MAX_L * 4];
    __shared__ double sh_shift;
    const int b = blockIdx.x, a = blockIdx.y;
    const int ld = L + 1;
    const size_t n = (size_t)ld * ld * F;
    const float* src = I_raw + (size_t)b * n;
    float* dst = I_out + ((size_t)b * n_alpha + a) * n;
    for (int x = threadIdx.x; x < L * F; x += SH_NT) {
        const int i = x / F, f = x - i * F;
        d[x] = src[((size_t)i * ld + (i + 1)) * F + f];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sum = 0.0;
        int count = 0;
        for (int x = 0; x < L * F; ++x) {
            const float v = d[x];
            if (v - v == 0.0f) {             // finite
                sum += (double)v;
                ++count;
            }
        }
        const double mean = count > 0 ? sum / (double)count : 0.0;
        sh_shift = (double)alpha[a] * mean;
        if (mean_out && a == 0) mean_out[b] = mean;
    }
    __syncthreads();
    const double shift = sh_shift;
    for (size_t x = threadIdx.x; x < n; x += SH_NT) dst[x] = (float)((double)src[x] - shift);
}

hipError_t launch_importance_shift(int B, int L, int F, int n_alpha, const float* I_raw,
                                   const float* alpha, float* I_out, double* mean_out,
                                   hipStream_t st)
{
    hipLaunchKernelGGL(importance_shift_kernel, dim3(B, n_alpha), dim3(SH_NT), 0, st, L, F, n_alpha,
                       I_raw, alpha, I_out, mean_out);
    return hipGetLastError();
}

// ---- trade-off curve -----------------------------------------------------------
// One workgroup per instance walks the row in chunks of FR_NT columns; a column
// is a point of the curve when its value exceeds that of the column before it.
// Points are numbered by a wave ballot, a prefix over the waves of the chunk
// and a running total, so they come out in ascending order of the budget.
constexpr int FR_NT = 256;

__global__ __launch_bounds__(FR_NT) void front_kernel(
    int L, int P, const float* __restrict__ M, int cap, int32_t* __restrict__ front_t,
    float* __restrict__ front_obj, int32_t* __restrict__ front_len)
{
    __shared__ int wave_count[FR_NT / 64];
    const int b = blockIdx.x;
    const float* row = M + ((size_t)b * (L + 1) + L) * P;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int total = 0;                                        // the same in every thread
    for (int t0 = 0; t0 < P; t0 += FR_NT) {
        const int t = t0 + threadIdx.x;
        float v = -INFINITY, below = -INFINITY;
        if (t < P) {
            v = row[t];
            if (t > 0) below = row[t - 1];
        }
        const bool point = v > below;
        const unsigned long long mask = __ballot(point);
        if (lane == 0) wave_count[wave] = __popcll(mask);
        __syncthreads();
        int before = total, all = 0;
#pragma unroll
        for (int w = 0; w < FR_NT / 64; ++w) {
            const int c = wave_count[w];
            if (w < wave) before += c;
            all += c;
        }
        if (point) {
            const int idx = before + __popcll(mask & ((1ull << lane) - 1ull));
            if (idx < cap) {
                front_t[(size_t)b * cap + idx] = t;
                front_obj[(size_t)b * cap + idx] = v;
            }
        }
        total += all;
        __syncthreads();                                  // wave_count is written again
    }
    if (threadIdx.x == 0) front_len[b] = total;
}

hipError_t launch_front(int B, int L, int P, const float* M, int cap, int32_t* front_t,
                        float* front_obj, int32_t* front_len, hipStream_t st)
{
    hipLaunchKernelGGL(front_kernel, dim3(B), dim3(FR_NT), 0, st, L, P, M, cap, front_t, front_obj,
                       front_len);
    return hipGetLastError();
}

// ---- the points of the curves as a query list -------------------------------------
// Instances are handled in tiles of 1024, FQ_SPLIT workgroups per tile.  Every
// workgroup first adds up the counts min(front_len, cap) of all earlier tiles
// (a strided sum, then one reduction), then scans the counts of its tile (wave
// scan, then the 16 wave totals), and copies its share of the tile's points,
// one list position per thread and pass (coalesced stores); the instance of a
// position is found by bisection of the tile's start offsets in LDS.
constexpr int FQ_SPLIT = 16;

__global__ __launch_bounds__(1024) void front_queries_kernel(
    int B, int cap, const int32_t* __restrict__ front_t, const int32_t* __restrict__ front_len,
    int qcap, int32_t* __restrict__ q_inst, int32_t* __restrict__ q_T0,
    int32_t* __restrict__ q_count)
{
    __shared__ long long red[16];
    __shared__ int wsum[16];
    __shared__ long long sstart[1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.y * 1024;
    // ---- points of the earlier tiles
    long long part = 0;
    for (int b = tid; b < b0; b += 1024) part += max(min(front_len[b], cap), 0);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int lo = __shfl_xor((int)(part & 0xFFFFFFFFll), d, 64);
        const int hi = __shfl_xor((int)(part >> 32), d, 64);
        part += ((long long)hi << 32) | (unsigned int)lo;
    }
    if (lane == 0) red[wave] = part;
    // ---- this tile
    const int b = b0 + tid;
    const int n = b < B ? max(min(front_len[b], cap), 0) : 0;
    int incl = n;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int v = __shfl_up(incl, d, 64);
        if (lane >= d) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    long long base = 0;
    int before = 0, tile = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        base += red[w];
        const int v = wsum[w];
        if (w < wave) before += v;
        tile += v;
    }
    sstart[tid] = base + before + incl - n;
    __syncthreads();
    for (long long q = base + (long long)blockIdx.x * 1024 + tid; q < base + tile && q < qcap;
         q += 1024 * FQ_SPLIT) {
        int lo = 0, hi = 1023;                            // the last instance that starts at or before q
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (sstart[mid] <= q) lo = mid; else hi = mid - 1;
        }
        q_inst[q] = b0 + lo;
        q_T0[q] = front_t[(size_t)(b0 + lo) * cap + (int)(q - sstart[lo])];
    }
    if (tid == 0 && blockIdx.x == 0 && blockIdx.y == gridDim.y - 1) {
        const long long total = base + tile;
        *q_count = (int32_t)(total > 0x7FFFFFFFll ? 0x7FFFFFFFll : total);
    }
}

hipError_t launch_front_queries(int B, int cap, const int32_t* front_t, const int32_t* front_len,
                                int qcap, int32_t* q_inst, int32_t* q_T0, int32_t* q_count,
                                hipStream_t st)
{
    const int ntiles = (B + 1023) / 1024;
    if (ntiles > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(front_queries_kernel, dim3(FQ_SPLIT, ntiles), dim3(1024), 0, st, B, cap,
                       front_t, front_len, qcap, q_inst, q_T0, q_count);
    return hipGetLastError();
}

// ---- latency of a network merged at a given set ---------------------------------
// One wave per query; lane x adds the blocks that end at members x, x + 64, ...
// of the chain 0 -> X -> L.  Latencies are non-negative, so the saturating
// left-to-right sum equals the exact 64-bit sum clamped once at the end.
constexpr int CL_WAVES = 4;

__global__ __launch_bounds__(64 * CL_WAVES) void chain_latency_kernel(
    int B, int L, const int32_t* __restrict__ T, int Q, const int32_t* __restrict__ q_inst,
    const int32_t* __restrict__ X, const int32_t* __restrict__ X_len, int32_t* __restrict__ lat)
{
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.x * CL_WAVES + (threadIdx.x >> 6);
    if (q >= Q) return;                                   // whole wave leaves together
    const int b = q_inst[q];
    const int n = X_len[q];
    if (b < 0 || b >= B || n < 0 || n > L - 1) {
        if (lane == 0) lat[q] = -1;
        return;
    }
    const int ld = L + 1;
    const int32_t* Tb = T + (size_t)b * ld * ld;
    const int32_t* Xq = X + (size_t)q * L;
    long long total = 0;
    bool valid = true;
    for (int x = lane; x <= n; x += 64) {                 // block x ends at member x (or at L)
        const int from = x > 0 ? Xq[x - 1] : 0;
        const int to = x < n ? Xq[x] : L;
        // members ascend strictly inside [1, L-1]
        if (from < 0 || to <= from || to > L || (x < n && to == L)) valid = false;
        else total += Tb[from * ld + to];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int lo = __shfl_xor((int)(total & 0xFFFFFFFFll), d, 64);
        const int hi = __shfl_xor((int)(total >> 32), d, 64);
        total += ((long long)hi << 32) | (unsigned int)lo;
    }
    const bool all_valid = __ballot(!valid) == 0;
    if (lane == 0) lat[q] = !all_valid ? -1 : total >= DPC_INF ? DPC_INF : (int32_t)total;
}

hipError_t launch_chain_latency(int B, int L, const int32_t* T, int Q, const int32_t* q_inst,
                                const int32_t* X, const int32_t* X_len, int32_t* lat,
                                hipStream_t st)
{
    hipLaunchKernelGGL(chain_latency_kernel, dim3((Q + CL_WAVES - 1) / CL_WAVES),
                       dim3(64 * CL_WAVES), 0, st, B, L, T, Q, q_inst, X, X_len, lat);
    return hipGetLastError();
}

}  // namespace dpc
