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
    int32_t off[S2_R];             // maxs - Topt[i][j0+rr]; 0 where there is no candidate
    float imp[S2_R];               // I[i][j0+rr]; -inf where there is no candidate
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
// exists when i < j, j <= L and 0 <= Topt[i][j] < P.  Shifts are stored as
// offsets below the largest shift of the record, the position of the candidate
// inside the LDS window of row i; a missing candidate has importance -inf and
// so never wins whatever it is added to.
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
    int wv[S2_R];
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
        wv[rr] = w;
        rec.imp[rr] = imp;
    }
#pragma unroll
    for (int rr = 0; rr < S2_R; ++rr) rec.off[rr] = wv[rr] < 0 ? 0 : maxs - wv[rr];
    const size_t idx = ((size_t)b * NR + r) * ld + i;
    recs[idx] = rec;
    infos[idx].mins = mins;
    infos[idx].maxs = maxs;
}

// Optional phase timers (build with -DDPC_S2_TIMERS): thread 0 of every
// workgroup accumulates wall-clock ticks (100 MHz) per phase and adds them to
// the spare words of the workspace header.
#ifdef DPC_S2_TIMERS
#define TMARK(var) const long long var = wall_clock64()
#define TACC(slot, a, b) do { if (tid == 0) tacc[slot] += (b) - (a); } while (0)
#else
#define TMARK(var) do {} while (0)
#define TACC(slot, a, b) do {} while (0)
#endif

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
// tp < 0, nothing for tp >= tlimit.  The window is cut into 16-byte groups, one
// per lane and pass.  A group inside [0, tlimit) goes global -> LDS without
// passing registers (the lanes of a wave fill consecutive 16-byte cells from a
// wave-uniform LDS base); a group entirely below 0 is one 16-byte store of
// -inf; the at most two groups that straddle 0 or tlimit are written element
// by element.  `row0`: the row is the base case M[0][t] = +0, not read from
// memory.
template <int NT, int SLOTW>
__device__ __forceinline__ void stage_window(float* slot, const float* row, int lo, int n,
                                             int tlimit, bool row0, int tid, int wave_base)
{
    constexpr int NGK = (SLOTW / 4 + NT - 1) / NT;
    constexpr float NINF = -INFINITY;
#pragma unroll
    for (int k = 0; k < NGK; ++k) {
        const int x = 4 * (tid + NT * k);
        const int tp = lo + x;
        if (x < n) {
            if (!row0 && tp >= 0 && tp + 3 < tlimit) {
                __builtin_amdgcn_global_load_lds(row + tp,
                                                 (lds_void*)(slot + 4 * (wave_base + NT * k)), 16,
                                                 0, 0);
            } else if (tp + 3 < 0) {
                *(float4*)(slot + x) = make_float4(NINF, NINF, NINF, NINF);
            } else if (row0 && tp >= 0) {
                *(float4*)(slot + x) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int tpe = tp + e;
                    if (tpe < tlimit) {
                        float v = NINF;
                        if (tpe >= 0) v = row0 ? 0.0f : row[tpe];
                        slot[x + e] = v;
                    }
                }
            }
        }
    }
}

template <int NT, int U, int CH, int DMAX, int WPE, bool STORE_K>
__global__ __launch_bounds__(NT, WPE) void stage2_tiled_kernel(
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

#ifdef DPC_S2_TIMERS
    long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const long long tkernel0 = wall_clock64();
#endif
    for (;;) {
        if (tid == 0) sh_word = (int)atomicAdd(&hdr->ticket, 1u);
        __syncthreads();
        const int ticket = __builtin_amdgcn_readfirstlane(sh_word);
        __syncthreads();
#ifdef DPC_S2_TIMERS
        if (ticket >= total && tid == 0) {
            tacc[7] = wall_clock64() - tkernel0;
            for (int q = 0; q < 8; ++q)
                atomicAdd((unsigned long long*)&hdr->pad[2 + 2 * q], (unsigned long long)tacc[q]);
            atomicAdd(&hdr->pad[20], 1u);
        }
#endif
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
            auto stage_chunk = [&](float (*buf)[SLOTW], int i0, const S2Info (&inf)[CH]) {
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = i0 + c;
                    const int mins = inf[c].mins, maxs = inf[c].maxs;
                    if (i < j0 && maxs >= 0 && maxs - mins <= DMAX && mins <= tmax) {
                        const int lo = t0 - maxs;
                        const int n = tend - mins - lo;
                        stage_window<NT, SLOTW>(buf[c], Mb + (size_t)i * P, lo, n, P, i == 0, tid,
                                                wave_base);
                    }
                }
            };

            // relax the block's rows from the rows [i0, i0+CH) held in `buf`
            auto relax_chunk = [&](const float (*buf)[SLOTW], int i0, const S2Rec (&rec)[CH],
                                   const S2Info (&inf)[CH]) {
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = i0 + c;
                    const int mins = inf[c].mins, maxs = inf[c].maxs;
                    if (i >= j0 || maxs < 0 || mins > tmax) continue;   // nothing reaches this strip
                    const int thr = maxs - tmax;       // candidate rr is in reach iff off >= thr
                    if (maxs - mins <= DMAX) {
                        // LDS reads run one row of the block ahead of the arithmetic
                        float mcur[U], mnxt[U];
                        auto fetch = [&](float (&m)[U], int rr) {
                            const bool ok = rec[c].off[rr] >= thr;
                            const int off = ok ? rec[c].off[rr] : 0;
                            const float* sp = &buf[c][off + tid];
#pragma unroll
                            for (int u = 0; u < U; ++u) m[u] = sp[NT * u];
                        };
                        fetch(mcur, 0);
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            if (rr + 1 < R) fetch(mnxt, rr + 1);
                            const bool ok = rec[c].off[rr] >= thr;
                            // select on the bit pattern: keeps the choice on the scalar unit
                            const float imp = __int_as_float(
                                ok ? __float_as_int(rec[c].imp[rr]) : (int)0xFF800000);
                            float cand[U];
                            bool win[U];
#pragma unroll
                            for (int u = 0; u < U; ++u) cand[u] = mcur[u] + imp;
#pragma unroll
                            for (int u = 0; u < U; ++u) win[u] = cand[u] > best[rr][u];
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                best[rr][u] = win[u] ? cand[u] : best[rr][u];
                                arg[rr][u] = win[u] ? i : arg[rr][u];
                            }
#pragma unroll
                            for (int u = 0; u < U; ++u) mcur[u] = mnxt[u];
                        }
                    } else {
                        const float* row = Mb + (size_t)i * P;
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            const int w = maxs - rec[c].off[rr];
                            if (w > tmax) continue;
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const int t = t0 + tid + NT * u;
                                if (t < P && t >= w) {
                                    const float m = (i == 0) ? 0.0f : row[t - w];
                                    const float cand = m + rec[c].imp[rr];
                                    if (cand > best[rr][u]) { best[rr][u] = cand; arg[rr][u] = i; }
                                }
                            }
                        }
                    }
                }
            };

            // one chunk: fetch its records and the next chunk's window extents (one
            // batch of scalar loads, in flight across the barrier), start the next
            // chunk's window copies, relax this chunk
            S2Info inf_cur[CH], inf_nxt[CH];
            auto load_infos = [&](S2Info (&inf)[CH], int i0) {
#pragma unroll
                for (int c = 0; c < CH; ++c) inf[c] = binfo[min(i0 + c, L)];
            };
            auto chunk_step = [&](float (*cur)[SLOTW], float (*nxt)[SLOTW], int i0) {
                S2Rec rec[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) rec[c] = brec[min(i0 + c, L)];
                load_infos(inf_nxt, i0 + CH);
                TMARK(ta);
                wait_lds_loads();
                __syncthreads();                       // `cur` filled, `nxt` free
                TMARK(tb);
                if (i0 + CH < j0) stage_chunk(nxt, i0 + CH, inf_nxt);
                TMARK(tc);
                relax_chunk(cur, i0, rec, inf_cur);
                TMARK(td);
                TACC(0, ta, tb);
                TACC(1, tb, tc);
                TACC(2, tc, td);
#pragma unroll
                for (int c = 0; c < CH; ++c) inf_cur[c] = inf_nxt[c];
            };

            // ---------------- off-diagonal part: rows i < j0 ----------------
            // (the barrier that ended the previous block's diagonal part, or the
            //  ticket barrier, has freed both buffers)
            load_infos(inf_cur, 0);
            stage_chunk(bufA, 0, inf_cur);
            for (int i0 = 0; i0 < j0; i0 += 2 * CH) {
                chunk_step(bufA, bufB, i0);
                if (i0 + CH < j0) chunk_step(bufB, bufA, i0 + CH);
            }

            // ---------------- diagonal part: rows inside the block ----------------
            // the strips to the left must have finished this block
            TMARK(te);
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
            TMARK(tf);
            TACC(3, te, tf);

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
                            const int w = hd[rr] - rec.off[r2];
                            const float imp = rec.imp[r2];
                            if (w > tmax) continue;
                            if (in_lds) {
                                const float* sp = &slot[rec.off[r2] + tid];
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
            TMARK(tg);
            TACC(4, tf, tg);
            if (s + 1 < NS) {
                __threadfence();
                __syncthreads();
                if (tid == 0)
                    __hip_atomic_store(my_flag, (uint32_t)(r + 1), __ATOMIC_RELEASE,
                                       __HIP_MEMORY_SCOPE_AGENT);
            } else {
                __syncthreads();                       // both buffers free for the next block
            }
            TMARK(th);
            TACC(5, tg, th);
        }
    }
}

template <int NT, int U, int CH, int DMAX, int WPE>
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

    // resident workgroups per compute unit: WPE waves per SIMD, 4 SIMDs
    constexpr int wg_per_cu = (WPE * 4 * 64) / NT;
    static_assert(wg_per_cu >= 1, "a workgroup must fit one compute unit");
    const int grid = (int)std::min<long long>(total, (long long)num_cu * wg_per_cu);
    const long long wait_limit = 500000000LL;      // 5 s of the 100 MHz wall clock
    if (K)
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, WPE, true>), dim3(grid), dim3(NT),
                           0, st, B, L, P, M, K, hdr, progress, recs, infos, NS, (int)total,
                           wait_limit);
    else
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, WPE, false>), dim3(grid),
                           dim3(NT), 0, st, B, L, P, M, K, hdr, progress, recs, infos, NS,
                           (int)total, wait_limit);
    return hipGetLastError();
}

int g_s2_shape = 0;     // tuning override, see launch_stage2_tiled

hipError_t launch_stage2_tiled(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                               uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    // strip width W = NT*U.  Narrow tables take the narrowest strip that covers
    // them; wide ones take the strip that gives about one workgroup-sized task
    // per resident slot, so that the strips of an instance run as one shallow
    // pipeline.
    int shape = g_s2_shape;
    if (shape == 0) {
        if (P <= 256) shape = 1;
        else if (P <= 512) shape = 2;
        else shape = 4;
    }
    switch (shape) {
        case 1: return launch_cfg<256, 1, 4, 240, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 2: return launch_cfg<256, 2, 4, 240, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 3: return launch_cfg<256, 4, 4, 256, 3>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 4: return launch_cfg<512, 2, 4, 256, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 5: return launch_cfg<1024, 2, 4, 256, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        default: return hipErrorInvalidValue;
    }
}

int stage2_tiled_error(const void* workspace_host_copy)
{
    return (int)((const S2Header*)workspace_host_copy)->error;
}

}  // namespace dpc
