// Stage 2, persistent LDS-tiled family (Algorithm 2 / recurrence Eq. 7 of the
// paper): M[j][t] = max_i fl32(M[i][t - Topt[i][j]] + I[i][j]), lowest arg-max.
//
// Decomposition.  The budget axis of one instance is cut into strips of W
// columns; the rows 1..L into blocks of R rows.  One workgroup owns a strip
// and walks its row blocks from top to bottom, keeping the R x W running
// (maximum, arg-max) pairs of the block in registers: lane `tid` owns the
// columns t0 + tid + NT*u, u < U, of every row of the block.
//
//   off-diagonal part  predecessors i below the block.  Row i is read through
//     a window [t0 - maxshift_i, t0 + W - minshift_i) staged once in LDS and
//     then used by all R rows of the block, each at its own wave-uniform
//     offset; consecutive lanes read consecutive LDS words.  Topt[i][j] and
//     I[i][j] are wave-uniform scalars.
//   diagonal part      predecessors inside the block, one row after the other:
//     a finished row is written to global memory and, together with a halo
//     fetched from the strips to its left, to an LDS slot from which the rows
//     below it in the block are relaxed.
//
// Dependencies point to lower rows and to lower-or-equal t only, so strip s
// needs, from the strips to its left, rows that are complete through the
// current block.  Strips are handed out as tickets in strip-major order by an
// atomic counter; a workgroup publishes "blocks completed" per (instance,
// strip) with release semantics and its right neighbour acquires it before
// the diagonal part of the same block.  Every ticket only waits on a lower
// ticket, which a running workgroup already owns, so the scheme cannot
// deadlock whatever the number of resident workgroups; the waits are
// time-bounded and a time-out makes every workgroup leave.
//
// A row whose shifts into the block spread over more than DMAX columns does
// not fit a slot; its candidates are read straight from global memory instead
// (same arithmetic, same order).
#include <algorithm>
#include "dpc_internal.h"

namespace dpc {

struct S2Workspace {
    uint32_t ticket;
    uint32_t error;
    uint32_t pad[62];
    uint32_t progress[1];      // [B * NS], blocks completed per (instance, strip)
};

__global__ void stage2_clear_kernel(uint32_t* w, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0;
}

hipError_t launch_clear_words(void* p, int nwords, hipStream_t st)
{
    hipLaunchKernelGGL(stage2_clear_kernel, dim3((nwords + 255) / 256), dim3(256), 0, st,
                       (uint32_t*)p, nwords);
    return hipGetLastError();
}

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NT, int U, int R, int DMAX, bool STORE_K>
__global__ __launch_bounds__(NT) void stage2_tiled_kernel(
    int B, int L, int P, const int32_t* __restrict__ Topt, const float* __restrict__ I, float* M,
    uint8_t* K, S2Workspace* ws, int NS, int total, long long wait_limit)
{
    constexpr int W = NT * U;
    constexpr int SLOTW = W + DMAX;
    constexpr float NINF = -INFINITY;
    __shared__ float slots[R][SLOTW];
    __shared__ int sh_word;

    const int tid = threadIdx.x;
    const int ld = L + 1;
    const int NR = (L + R - 1) / R;

    for (;;) {
        if (tid == 0) sh_word = (int)atomicAdd(&ws->ticket, 1u);
        __syncthreads();
        const int ticket = __builtin_amdgcn_readfirstlane(sh_word);
        __syncthreads();
        if (ticket >= total) return;
        const int s = ticket / B;
        const int b = ticket - s * B;
        const int t0 = s * W;
        const int tend = min(t0 + W, P);
        const int tmax = tend - 1;
        const int32_t* To = Topt + (size_t)b * ld * ld;
        const float* Ib = I + (size_t)b * ld * ld;
        float* Mb = M + (size_t)b * ld * P;
        uint8_t* Kb = STORE_K ? K + (size_t)b * ld * P : nullptr;
        uint32_t* my_flag = &ws->progress[(size_t)b * NS + s];

        // row 0: the base case
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + tid + NT * u;
            if (t < P) {
                Mb[t] = 0.0f;
                if (STORE_K) Kb[t] = DPC_NOARG;
            }
        }

        for (int r = 0; r < NR; ++r) {
            const int j0 = 1 + r * R;
            const int rcur = min(R, ld - j0);
            float best[R][U];
            int arg[R][U];
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
#pragma unroll
                for (int u = 0; u < U; ++u) { best[rr][u] = NINF; arg[rr][u] = DPC_NOARG; }

            // ---------------- off-diagonal part: rows i < j0 ----------------
            for (int i0 = 0; i0 < j0; i0 += R) {
                const int nrow = min(R, j0 - i0);
                __syncthreads();                       // slots free again
                for (int c = 0; c < nrow; ++c) {
                    const int i = i0 + c;
                    int mins = 0x7FFFFFFF, maxs = -1;
#pragma unroll
                    for (int rr = 0; rr < R; ++rr) {
                        const int w = To[i * ld + min(j0 + rr, L)];
                        if (rr < rcur && (unsigned)w <= (unsigned)tmax) {
                            mins = min(mins, w);
                            maxs = max(maxs, w);
                        }
                    }
                    if (maxs >= 0 && maxs - mins <= DMAX) {
                        const int lo = t0 - maxs;
                        const int len = tend - mins - lo;
                        const float* row = Mb + (size_t)i * P;
                        for (int x = tid; x < len; x += NT) {
                            const int tp = lo + x;
                            float v = NINF;
                            if (tp >= 0) v = (i == 0) ? 0.0f : row[tp];
                            slots[c][x] = v;
                        }
                    }
                }
                __syncthreads();                       // slots filled
                for (int c = 0; c < nrow; ++c) {
                    const int i = i0 + c;
                    int wv[R];
                    float iv[R];
                    int mins = 0x7FFFFFFF, maxs = -1;
#pragma unroll
                    for (int rr = 0; rr < R; ++rr) {
                        const int jj = min(j0 + rr, L);
                        int w = To[i * ld + jj];
                        float imp = Ib[i * ld + jj];
                        if (!(rr < rcur && (unsigned)w <= (unsigned)tmax)) { w = -1; imp = NINF; }
                        else { mins = min(mins, w); maxs = max(maxs, w); }
                        wv[rr] = w;
                        iv[rr] = imp;
                    }
                    if (maxs < 0) continue;            // no candidate reaches this strip
                    if (maxs - mins <= DMAX) {
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            const int off = wv[rr] < 0 ? 0 : maxs - wv[rr];
                            const float imp = iv[rr];
                            const float* sp = &slots[c][off + tid];
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const float cand = sp[NT * u] + imp;
                                if (cand > best[rr][u]) { best[rr][u] = cand; arg[rr][u] = i; }
                            }
                        }
                    } else {
                        const float* row = Mb + (size_t)i * P;
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            if (wv[rr] < 0) continue;
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const int t = t0 + tid + NT * u;
                                if (t < P && t >= wv[rr]) {
                                    const float m = (i == 0) ? 0.0f : row[t - wv[rr]];
                                    const float cand = m + iv[rr];
                                    if (cand > best[rr][u]) { best[rr][u] = cand; arg[rr][u] = i; }
                                }
                            }
                        }
                    }
                }
            }

            // ---------------- diagonal part: rows inside the block ----------------
            // the strips to the left must have finished this block
            if (s > 0) {
                if (tid == 0) {
                    const uint32_t* flag = &ws->progress[(size_t)b * NS + s - 1];
                    const long long start = wall_clock64();
                    int ok = 1;
                    while (ld_relaxed(flag) < (uint32_t)(r + 1)) {
                        if (ld_relaxed(&ws->error) != 0) { ok = 0; break; }
                        if (wall_clock64() - start > wait_limit) {
                            __hip_atomic_store(&ws->error, 1u, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                            ok = 0;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(4);
                    }
                    sh_word = ok;
                }
                __syncthreads();
                const int ok = __builtin_amdgcn_readfirstlane(sh_word);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                if (!ok) return;                       // uniform: every thread leaves
            }
            __syncthreads();                           // off-diagonal readers done; sh_word free

            // halo of every row of the block that feeds a later row of the block
            int hd[R];
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                hd[rr] = -1;
                if (rr + 1 < rcur) {
                    const int j = j0 + rr;
#pragma unroll
                    for (int r2 = rr + 1; r2 < R; ++r2) {
                        const int w = To[j * ld + min(j0 + r2, L)];
                        if (r2 < rcur && (unsigned)w <= (unsigned)tmax) hd[rr] = max(hd[rr], w);
                    }
                    if (hd[rr] >= 0 && hd[rr] <= DMAX) {
                        const float* row = Mb + (size_t)j * P;
                        for (int x = tid; x < hd[rr]; x += NT) {
                            const int tp = t0 - hd[rr] + x;
                            slots[rr][x] = tp >= 0 ? row[tp] : NINF;
                        }
                    }
                }
            }

#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const int j = j0 + rr;
                if (rr < rcur) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int t = t0 + tid + NT * u;
                        if (t < P) {
                            Mb[(size_t)j * P + t] = best[rr][u];
                            if (STORE_K) Kb[(size_t)j * P + t] = (uint8_t)arg[rr][u];
                        }
                    }
                    if (hd[rr] >= 0 && hd[rr] <= DMAX) {
#pragma unroll
                        for (int u = 0; u < U; ++u) slots[rr][hd[rr] + tid + NT * u] = best[rr][u];
                    }
                }
                if (rr + 1 < R) {
                    __syncthreads();                   // row j visible: LDS slot and global
                    if (hd[rr] >= 0) {
                        const bool in_lds = hd[rr] <= DMAX;
                        const float* row = Mb + (size_t)j * P;
#pragma unroll
                        for (int r2 = rr + 1; r2 < R; ++r2) {
                            const int jj = min(j0 + r2, L);
                            const int w = To[j * ld + jj];
                            const float imp = Ib[j * ld + jj];
                            if (!(r2 < rcur && (unsigned)w <= (unsigned)tmax)) continue;
                            if (in_lds) {
                                const float* sp = &slots[rr][hd[rr] - w + tid];
#pragma unroll
                                for (int u = 0; u < U; ++u) {
                                    const float cand = sp[NT * u] + imp;
                                    if (cand > best[r2][u]) { best[r2][u] = cand; arg[r2][u] = j; }
                                }
                            } else {
#pragma unroll
                                for (int u = 0; u < U; ++u) {
                                    const int t = t0 + tid + NT * u;
                                    if (t < P && t >= w) {
                                        const float cand = row[t - w] + imp;
                                        if (cand > best[r2][u]) { best[r2][u] = cand; arg[r2][u] = j; }
                                    }
                                }
                            }
                        }
                    }
                }
            }

            // publish: this strip has finished block r
            if (s + 1 < NS) {
                __threadfence();
                __syncthreads();
                if (tid == 0)
                    __hip_atomic_store(my_flag, (uint32_t)(r + 1), __ATOMIC_RELEASE,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
    }
}

size_t stage2_tiled_workspace_bytes(int B, int L, int P)
{
    (void)L;
    const size_t ns = ((size_t)P + 255) / 256;     // upper bound over every strip width used
    size_t n = sizeof(S2Workspace) + 4 * (size_t)B * ns;
    return (n + 255) & ~(size_t)255;
}

template <int NT, int U, int R, int DMAX>
static hipError_t launch_cfg(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                             uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    constexpr int W = NT * U;
    const int NS = (P + W - 1) / W;
    const long long total = (long long)B * NS;
    if (total > 0x7FFFFFF0LL) return hipErrorInvalidValue;
    S2Workspace* ws = (S2Workspace*)workspace;
    const int nwords = (int)(sizeof(S2Workspace) / 4) + B * NS;
    hipError_t e = launch_clear_words(workspace, nwords, st);
    if (e != hipSuccess) return e;
    const int wg_per_cu = 2;
    const int grid = (int)std::min<long long>(total, (long long)num_cu * wg_per_cu);
    const long long wait_limit = 500000000LL;      // 5 s of the 100 MHz wall clock
    if (K)
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, R, DMAX, true>), dim3(grid), dim3(NT), 0, st,
                           B, L, P, Topt, I, M, K, ws, NS, (int)total, wait_limit);
    else
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, R, DMAX, false>), dim3(grid), dim3(NT), 0,
                           st, B, L, P, Topt, I, M, K, ws, NS, (int)total, wait_limit);
    return hipGetLastError();
}

hipError_t launch_stage2_tiled(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                               uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    if (P <= 256) return launch_cfg<256, 1, 8, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
    if (P <= 512) return launch_cfg<256, 2, 8, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
    return launch_cfg<256, 4, 8, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
}

int stage2_tiled_error(const void* workspace_host_copy)
{
    return (int)((const S2Workspace*)workspace_host_copy)->error;
}

}  // namespace dpc
