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
//     a window [t0 - maxshift_i, t0 + W - minshift_i) copied once into an LDS
//     slot (global -> LDS loads that bypass the registers, 16 bytes per lane)
//     and then used by all R rows of the block, each at its own wave-uniform
//     offset; consecutive lanes read consecutive LDS words.  The slots form
//     two buffers of CH rows: while one chunk of rows is relaxed the next is
//     in flight.
//   diagonal part      predecessors inside the block, one row after the other:
//     a finished row is written to global memory and, together with a halo
//     fetched from the strips to its left, to an LDS slot from which the rows
//     below it in the block are relaxed.
//
// Topt and I are first repacked per (instance, row block, predecessor i) into
// 64-byte records {shift[R], importance[R]} plus the minimum and maximum shift,
// so that the wave-uniform operands of a whole row arrive with one scalar load.
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

typedef __attribute__((address_space(3))) void lds_void;

constexpr int S2_R = 8;            // rows per block (record layout depends on it)

struct S2Header {
    uint32_t ticket;
    uint32_t error;
    uint32_t pad[62];
};

struct __attribute__((aligned(64))) S2Rec {
    int32_t w[S2_R];               // shift Topt[i][j0+rr]; -1 = no candidate
    float imp[S2_R];               // I[i][j0+rr]; -inf where w = -1
};

struct S2Info {
    int32_t mins, maxs;            // over the valid shifts of the record; maxs = -1: none
};

struct S2Layout {
    size_t progress_off, rec_off, info_off, total;
};

static S2Layout s2_layout(int B, int L, int P)
{
    S2Layout l;
    const size_t ns = ((size_t)P + 255) / 256;      // upper bound over every strip width used
    const size_t nr = ((size_t)L + S2_R - 1) / S2_R;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    l.progress_off = sizeof(S2Header);
    l.rec_off = up(l.progress_off + 4 * (size_t)B * ns);
    l.info_off = up(l.rec_off + sizeof(S2Rec) * (size_t)B * nr * (L + 1));
    l.total = up(l.info_off + sizeof(S2Info) * (size_t)B * nr * (L + 1));
    return l;
}

size_t stage2_tiled_workspace_bytes(int B, int L, int P) { return s2_layout(B, L, P).total; }

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

// One record per (instance b, row block r, predecessor i): the candidates that
// row i offers to the rows j0..j0+R-1 of block r (j0 = 1 + r*R).  A candidate
// exists when i < j, j <= L and 0 <= Topt[i][j] < P.
__global__ __launch_bounds__(256) void stage2_pack_kernel(
    int L, int P, int NR, const int32_t* __restrict__ Topt, const float* __restrict__ I,
    S2Rec* __restrict__ recs, S2Info* __restrict__ infos)
{
    const int ld = L + 1;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    const int b = blockIdx.z;
    if (i >= ld) return;
    const int j0 = 1 + r * S2_R;
    const int32_t* To = Topt + (size_t)b * ld * ld;
    const float* Ib = I + (size_t)b * ld * ld;
    S2Rec rec;
    int mins = 0x7FFFFFFF, maxs = -1;
#pragma unroll
    for (int rr = 0; rr < S2_R; ++rr) {
        const int j = j0 + rr;
        int w = -1;
        float imp = -INFINITY;
        if (j <= L && i < j) {
            const int v = To[i * ld + j];
            if (v >= 0 && v < P) {
                w = v;
                imp = Ib[i * ld + j];
                mins = min(mins, w);
                maxs = max(maxs, w);
            }
        }
        rec.w[rr] = w;
        rec.imp[rr] = imp;
    }
    const size_t idx = ((size_t)b * NR + r) * ld + i;
    recs[idx] = rec;
    infos[idx].mins = mins;
    infos[idx].maxs = maxs;
}

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// wait until every global -> LDS load this wave has issued has landed
__device__ __forceinline__ void wait_lds_loads()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0), expcnt and lgkmcnt untouched
}

// Copy the window tp in [lo, lo + n) of a row of M into slot[0..n): -inf for
// tp < 0, nothing for tp >= tlimit.  16-byte groups that lie inside
// [0, tlimit) go global -> LDS without passing registers (the lanes of a wave
// fill consecutive 16-byte cells from a wave-uniform LDS base); the groups at
// the edges are written element by element.  `row0`: the row is the base case
// M[0][t] = +0, not read from memory.
template <int NT, int SLOTW>
__device__ __forceinline__ void stage_window(float* slot, const float* row, int lo, int n,
                                             int tlimit, bool row0, int tid, int wave_base)
{
    constexpr int NGK = (SLOTW / 4 + NT - 1) / NT;
#pragma unroll
    for (int k = 0; k < NGK; ++k) {
        const int x = 4 * (tid + NT * k);
        const int tp = lo + x;
        if (x < n) {
            if (!row0 && tp >= 0 && tp + 3 < tlimit) {
                __builtin_amdgcn_global_load_lds(row + tp,
                                                 (lds_void*)(slot + 4 * (wave_base + NT * k)), 16,
                                                 0, 0);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int tpe = tp + e;
                    if (tpe < tlimit) {
                        float v = -INFINITY;
                        if (tpe >= 0) v = row0 ? 0.0f : row[tpe];
                        slot[x + e] = v;
                    }
                }
            }
        }
    }
}

template <int NT, int U, int CH, int DMAX, bool STORE_K>
__global__ __launch_bounds__(NT) void stage2_tiled_kernel(
    int B, int L, int P, float* M, uint8_t* K, S2Header* hdr, uint32_t* progress,
    const S2Rec* __restrict__ recs, const S2Info* __restrict__ infos, int NS, int total,
    long long wait_limit)
{
    constexpr int R = S2_R;
    constexpr int W = NT * U;
    constexpr int SLOTW = W + DMAX + 4;     // multiple of 4
    constexpr float NINF = -INFINITY;
    static_assert(2 * CH >= R - 1, "the diagonal part needs R-1 slots");
    __shared__ __attribute__((aligned(16))) float bufA[CH][SLOTW];
    __shared__ __attribute__((aligned(16))) float bufB[CH][SLOTW];
    __shared__ int sh_word;

    const int tid = threadIdx.x;
    const int wave_base = __builtin_amdgcn_readfirstlane(tid & ~63);
    const int ld = L + 1;
    const int NR = (L + R - 1) / R;

    for (;;) {
        if (tid == 0) sh_word = (int)atomicAdd(&hdr->ticket, 1u);
        __syncthreads();
        const int ticket = __builtin_amdgcn_readfirstlane(sh_word);
        __syncthreads();
        if (ticket >= total) return;
        const int s = ticket / B;
        const int b = ticket - s * B;
        const int t0 = s * W;
        const int tend = min(t0 + W, P);
        const int tmax = tend - 1;
        float* Mb = M + (size_t)b * ld * P;
        uint8_t* Kb = STORE_K ? K + (size_t)b * ld * P : nullptr;
        uint32_t* my_flag = &progress[(size_t)b * NS + s];

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
            const S2Rec* brec = recs + ((size_t)b * NR + r) * ld;
            const S2Info* binfo = infos + ((size_t)b * NR + r) * ld;
            float best[R][U];
            int arg[R][U];
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
#pragma unroll
                for (int u = 0; u < U; ++u) { best[rr][u] = NINF; arg[rr][u] = DPC_NOARG; }

            // stage the windows of rows [i0, i0+CH) into `buf` (asynchronous)
            auto stage_chunk = [&](float (*buf)[SLOTW], int i0) {
                const int nrow = min(CH, j0 - i0);
                for (int c = 0; c < nrow; ++c) {
                    const int i = i0 + c;
                    const int mins = binfo[i].mins, maxs = binfo[i].maxs;
                    if (maxs >= 0 && maxs - mins <= DMAX && mins <= tmax) {
                        const int lo = t0 - maxs;
                        const int n = tend - mins - lo;
                        stage_window<NT, SLOTW>(buf[c], Mb + (size_t)i * P, lo, n, P, i == 0, tid,
                                                wave_base);
                    }
                }
            };

            // relax the block's rows from the rows [i0, i0+CH) held in `buf`
            auto relax_chunk = [&](const float (*buf)[SLOTW], int i0) {
                const int nrow = min(CH, j0 - i0);
                for (int c = 0; c < nrow; ++c) {
                    const int i = i0 + c;
                    const S2Rec rec = brec[i];
                    const int mins = binfo[i].mins, maxs = binfo[i].maxs;
                    if (maxs < 0 || mins > tmax) continue;     // nothing reaches this strip
                    if (maxs - mins <= DMAX) {
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            const bool ok = (unsigned)rec.w[rr] <= (unsigned)tmax;
                            const int off = ok ? maxs - rec.w[rr] : 0;
                            // select on the bit pattern: keeps the choice on the scalar unit
                            const float imp = __int_as_float(
                                ok ? __float_as_int(rec.imp[rr]) : (int)0xFF800000);
                            const float* sp = &buf[c][off + tid];
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
                            const int w = rec.w[rr];
                            if ((unsigned)w > (unsigned)tmax) continue;
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const int t = t0 + tid + NT * u;
                                if (t < P && t >= w) {
                                    const float m = (i == 0) ? 0.0f : row[t - w];
                                    const float cand = m + rec.imp[rr];
                                    if (cand > best[rr][u]) { best[rr][u] = cand; arg[rr][u] = i; }
                                }
                            }
                        }
                    }
                }
            };

            // ---------------- off-diagonal part: rows i < j0 ----------------
            // (the barrier that ended the previous block's diagonal part, or the
            //  ticket barrier, has freed both buffers)
            stage_chunk(bufA, 0);
            for (int i0 = 0; i0 < j0; i0 += 2 * CH) {
                wait_lds_loads();
                __syncthreads();                       // bufA filled, bufB free
                if (i0 + CH < j0) stage_chunk(bufB, i0 + CH);
                relax_chunk(bufA, i0);
                if (i0 + CH < j0) {
                    wait_lds_loads();
                    __syncthreads();                   // bufB filled, bufA free
                    if (i0 + 2 * CH < j0) stage_chunk(bufA, i0 + 2 * CH);
                    relax_chunk(bufB, i0 + CH);
                }
            }

            // ---------------- diagonal part: rows inside the block ----------------
            // the strips to the left must have finished this block
            if (s > 0) {
                if (tid == 0) {
                    const uint32_t* flag = &progress[(size_t)b * NS + s - 1];
                    const long long start = wall_clock64();
                    int ok = 1;
                    while (ld_relaxed(flag) < (uint32_t)(r + 1)) {
                        if (ld_relaxed(&hdr->error) != 0) { ok = 0; break; }
                        if (wall_clock64() - start > wait_limit) {
                            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED,
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

            // halo [t0 - hd, t0) of every row of the block that feeds a later row
            int hd[R];
#pragma unroll
            for (int rr = 0; rr < R - 1; ++rr) {
                hd[rr] = -1;
                if (rr + 1 < rcur) {
                    const int j = j0 + rr;
                    const int mins = binfo[j].mins, maxs = binfo[j].maxs;
                    if (maxs >= 0 && mins <= tmax) {
                        hd[rr] = maxs;
                        if (maxs <= DMAX) {
                            float* slot = rr < CH ? bufA[rr] : bufB[rr - CH];
                            stage_window<NT, SLOTW>(slot, Mb + (size_t)j * P, t0 - maxs, maxs, t0,
                                                    false, tid, wave_base);
                        }
                    }
                }
            }
            hd[R - 1] = -1;
            wait_lds_loads();

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
                    if (rr < R - 1 && hd[rr] >= 0 && hd[rr] <= DMAX) {
                        float* slot = rr < CH ? bufA[rr] : bufB[rr - CH];
#pragma unroll
                        for (int u = 0; u < U; ++u) slot[hd[rr] + tid + NT * u] = best[rr][u];
                    }
                }
                if (rr + 1 < R) {
                    __syncthreads();                   // row j visible: LDS slot and global
                    if (hd[rr] >= 0) {
                        const S2Rec rec = brec[j];
                        const bool in_lds = hd[rr] <= DMAX;
                        const float* slot = rr < CH ? bufA[rr] : bufB[rr - CH];
                        const float* row = Mb + (size_t)j * P;
#pragma unroll
                        for (int r2 = rr + 1; r2 < R; ++r2) {
                            const int w = rec.w[r2];
                            const float imp = rec.imp[r2];
                            if ((unsigned)w > (unsigned)tmax) continue;
                            if (in_lds) {
                                const float* sp = &slot[hd[rr] - w + tid];
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
            } else {
                __syncthreads();                       // both buffers free for the next block
            }
        }
    }
}

template <int NT, int U, int CH, int DMAX>
static hipError_t launch_cfg(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                             uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    constexpr int W = NT * U;
    const int NS = (P + W - 1) / W;
    const int NR = (L + S2_R - 1) / S2_R;
    const long long total = (long long)B * NS;
    if (total > 0x7FFFFFF0LL) return hipErrorInvalidValue;
    const S2Layout lay = s2_layout(B, L, P);
    char* base = (char*)workspace;
    S2Header* hdr = (S2Header*)base;
    uint32_t* progress = (uint32_t*)(base + lay.progress_off);
    S2Rec* recs = (S2Rec*)(base + lay.rec_off);
    S2Info* infos = (S2Info*)(base + lay.info_off);

    const int nwords = (int)(sizeof(S2Header) / 4) + B * NS;
    hipError_t e = launch_clear_words(workspace, nwords, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stage2_pack_kernel, dim3((L + 1 + 255) / 256, NR, B), dim3(256), 0, st, L, P,
                       NR, Topt, I, recs, infos);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    const int wg_per_cu = 3;
    const int grid = (int)std::min<long long>(total, (long long)num_cu * wg_per_cu);
    const long long wait_limit = 500000000LL;      // 5 s of the 100 MHz wall clock
    if (K)
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, true>), dim3(grid), dim3(NT), 0,
                           st, B, L, P, M, K, hdr, progress, recs, infos, NS, (int)total,
                           wait_limit);
    else
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, false>), dim3(grid), dim3(NT), 0,
                           st, B, L, P, M, K, hdr, progress, recs, infos, NS, (int)total,
                           wait_limit);
    return hipGetLastError();
}

hipError_t launch_stage2_tiled(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                               uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    if (P <= 256) return launch_cfg<256, 1, 4, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
    if (P <= 512) return launch_cfg<256, 2, 4, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
    return launch_cfg<256, 4, 4, 256>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
}

int stage2_tiled_error(const void* workspace_host_copy)
{
    return (int)((const S2Header*)workspace_host_copy)->error;
}

}  // namespace dpc
