// Stage 2, persistent LDS-tiled family (Algorithm 2 / recurrence Eq. 7 of the
// paper): M[j][t] = max_i fl32(M[i][t - Topt[i][j]] + I[i][j]), lowest arg-max.
//
// Tasks.  The rows 1..L of an instance are cut into groups of R = 8 rows, the
// budget axis into strips.  One task = (instance, row group, strip); it reads
// only rows below its group from global memory and writes its own rows, so it
// carries no state from task to task.  A workgroup keeps the R x WCAP running
// (maximum, arg-max) pairs of a task in registers: lane `tid` owns the columns
// tS + tid + NT*u, u < U, of every row of the group.
//
//   off-diagonal part  predecessors i below the group.  Row i is read through a
//     window [tS - maxshift_i, tS + WCAP - minshift_i) copied once into an LDS
//     slot (global -> LDS loads that bypass the registers, 16 bytes per lane)
//     and then used by all R rows of the group, each at its own wave-uniform
//     offset; consecutive lanes read consecutive LDS words.  The slots form
//     two buffers of CH rows: while one chunk of rows is relaxed the next is
//     in flight.
//   diagonal part      predecessors inside the group, one row after the other:
//     a finished row goes to an LDS slot from which the rows below it in the
//     group are relaxed.
//
// Ghost columns.  Inside a group, row j needs row i of the same group at
// t - Topt[i][j], which for the first columns of a strip lies in the strip to
// the left.  Instead of waiting for that strip the task recomputes those
// columns itself: it starts g columns to the left of the columns it stores,
// g = the longest chain of shifts inside the group, so every stored cell only
// depends on cells the task computed correctly.  Tasks of one group are then
// independent of each other.
//
// Order.  Tasks are handed out as tickets by an atomic counter, level by level
// (level = row group), instance by instance, strip by strip.  A task waits for
// the completion counter of the previous level of its instance (release /
// acquire at agent scope); that level's tickets were all handed out one whole
// level earlier, so the wait is normally over before it starts, and it can
// never deadlock because it only ever waits on lower tickets.  Waits are
// time-bounded; a time-out makes every workgroup leave.
//
// Fallback.  If the shifts of some predecessor into a group spread over more
// than DMAX columns, or the ghost width of the group exceeds its limit, the
// group is run as R levels of one row each (spread 0, no ghost columns).
//
// Topt and I are first repacked per (instance, row group, predecessor i) into
// 64-byte records {offset[R], importance[R]} plus the minimum and maximum
// shift, so that the wave-uniform operands of a row arrive with one scalar
// load; a second small kernel lays out the task table.
#include <algorithm>
#include <type_traits>
#include "dpc_internal.h"

namespace dpc {

typedef __attribute__((address_space(3))) void lds_void;

constexpr int S2_R = 8;            // rows per group (record layout depends on it)

struct S2Header {
    uint32_t ticket;
    uint32_t error;
    uint32_t total;                // number of tasks, written by the layout kernel
    uint32_t pad[61];
};

struct __attribute__((aligned(64))) S2Rec {
    uint32_t offp[S2_R / 2];       // 4 * (maxs - Topt[i][j0+rr]) as 16-bit halves (rr even: low),
                                   // the byte offset of the candidate in the LDS window of row
                                   // i; 0 where there is no candidate
    float imp[S2_R];               // I[i][j0+rr]; -inf where there is no candidate
    uint32_t pad[S2_R / 2];
};

// byte offset of candidate rr inside the window of its row
__device__ __forceinline__ int rec_off4(const S2Rec& r, int rr)
{
    return (rr & 1) ? (int)(r.offp[rr >> 1] >> 16) : (int)(r.offp[rr >> 1] & 0xFFFFu);
}

struct S2Shift {
    int32_t w[S2_R];               // Topt[i][j0+rr] itself, -1 where there is no candidate
};                                 // (read by the row-by-row path only)

struct S2Info {
    int32_t mins, maxs;            // over the valid shifts of the record; maxs = -1: none
};

// one entry per (level, instance); level = group * R + row-in-group
struct S2Entry {
    int32_t cnt;                   // number of strips (tasks)
    int32_t prev;                  // entry that must be complete first, -1: none
    int32_t prev_cnt;              // number of tasks of that entry
    int32_t g;                     // >= 0: whole group, ghost width; -1: one row
};

struct S2Task {
    int32_t entry, strip;          // in ticket order
};

struct S2Layout {
    size_t done_off, entry_off, group_off, task_off, rec_off, info_off, shift_off, total;
    long long nentries, maxtasks;
};

static S2Layout s2_layout(int B, int L, int P)
{
    S2Layout l;
    const size_t nq = ((size_t)L + S2_R - 1) / S2_R;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    l.nentries = (long long)nq * S2_R * B;
    // most tasks arise when every group runs row by row with the narrowest strips
    l.maxtasks = l.nentries * (((long long)P + 255) / 256);
    l.done_off = sizeof(S2Header);
    l.entry_off = up(l.done_off + 4 * (size_t)l.nentries);
    l.group_off = up(l.entry_off + sizeof(S2Entry) * ((size_t)l.nentries + 1));
    l.task_off = up(l.group_off + 4 * (size_t)B * nq);
    l.rec_off = up(l.task_off + sizeof(S2Task) * (size_t)l.maxtasks);
    l.info_off = up(l.rec_off + sizeof(S2Rec) * (size_t)B * nq * (L + 1));
    l.shift_off = up(l.info_off + sizeof(S2Info) * (size_t)B * nq * (L + 1));
    l.total = up(l.shift_off + sizeof(S2Shift) * (size_t)B * nq * (L + 1));
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

// One record per (instance b, row group q, predecessor i): the candidates that
// row i offers to the rows j0..j0+R-1 of the group (j0 = 1 + q*R).  A candidate
// exists when i < j, j <= L and 0 <= Topt[i][j] < P.  Shifts are stored as
// offsets below the largest shift of the record, the position of the candidate
// inside the LDS window of row i; a missing candidate has importance -inf and
// so never wins whatever it is added to.  The workgroup also decides how the
// group runs: groups[b][q] = ghost width g if every spread and every shift
// inside the group fits dmax and g <= gmax, else -1 (row by row).
__global__ __launch_bounds__(256) void stage2_pack_kernel(
    int L, int P, int NQ, const int32_t* __restrict__ Topt, const float* __restrict__ I,
    S2Rec* __restrict__ recs, S2Info* __restrict__ infos, S2Shift* __restrict__ shifts,
    int32_t* __restrict__ groups, int gmax, int dmax, int wcap)
{
    __shared__ int wd[S2_R][S2_R];
    __shared__ int viol;
    const int ld = L + 1;
    const int i = threadIdx.x;             // L <= 255: one thread per predecessor
    const int q = blockIdx.x;
    const int b = blockIdx.y;
    const int j0 = 1 + q * S2_R;
    const int32_t* To = Topt + (size_t)b * ld * ld;
    const float* Ib = I + (size_t)b * ld * ld;
    if (i == 0) viol = 0;
    __syncthreads();
    S2Rec rec;
    int wv[S2_R];
    int mins = 0x7FFFFFFF, maxs = -1;
#pragma unroll
    for (int rr = 0; rr < S2_R; ++rr) {
        const int j = j0 + rr;
        int w = -1;
        float imp = -INFINITY;
        if (i < ld && j <= L && i < j) {
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
    for (int rr = 0; rr < S2_R / 2; ++rr) {
        // a spread beyond dmax sends the group to the row-by-row path, which does
        // not use these offsets: clamp so that the halves cannot overflow
        const uint32_t lo = wv[2 * rr] < 0 ? 0u : (uint32_t)min(maxs - wv[2 * rr], 16383) * 4u;
        const uint32_t hi = wv[2 * rr + 1] < 0 ? 0u : (uint32_t)min(maxs - wv[2 * rr + 1], 16383) * 4u;
        rec.offp[rr] = lo | (hi << 16);
        rec.pad[rr] = 0;
    }
    if (i < ld) {
        const size_t idx = ((size_t)b * NQ + q) * ld + i;
        recs[idx] = rec;
        infos[idx].mins = mins;
        infos[idx].maxs = maxs;
#pragma unroll
        for (int rr = 0; rr < S2_R; ++rr) shifts[idx].w[rr] = wv[rr];
    }
    if (i < j0 && maxs >= 0 && maxs - mins > dmax) viol = 1;
    if (i >= j0 && i < j0 + S2_R) {
#pragma unroll
        for (int rr = 0; rr < S2_R; ++rr) wd[i - j0][rr] = wv[rr];
    }
    __syncthreads();
    if (i == 0) {
        // how far to the left of its stored columns each row must be correct
        int need[S2_R];
        int g = 0, hmax = 0;
        for (int rr = S2_R - 1; rr >= 0; --rr) {
            int n = 0;
            for (int r2 = rr + 1; r2 < S2_R; ++r2)
                if (wd[rr][r2] >= 0) {
                    n = max(n, wd[rr][r2] + need[r2]);
                    hmax = max(hmax, wd[rr][r2]);
                }
            need[rr] = n;
            g = max(g, n);
        }
        // a table that fits one task has no strip to its left: no ghost columns
        const bool bad = viol || hmax > dmax || (P > wcap && g > gmax);
        groups[(size_t)b * NQ + q] = bad ? -1 : g;
    }
}

// Task table: entries in ticket order (level-major, then instance), the task
// list (entry and strip of every ticket) and the total.  One workgroup walks
// the entries in tiles of 1024, one entry per thread (so that its stores are
// coalesced), with a running prefix sum of the strip counts: wave scan, then
// one combine of the 16 wave totals per tile.  The per-group decisions are
// first brought into LDS when they fit.
constexpr int S2_LAYOUT_CACHE = 12288;
__global__ __launch_bounds__(1024) void stage2_layout_kernel(
    int B, int L, int P, int NQ, int wcap, const int32_t* __restrict__ groups,
    S2Entry* __restrict__ entries, S2Task* __restrict__ tasks, S2Header* hdr)
{
    __shared__ int wsum[2][16];
    __shared__ int gcache[S2_LAYOUT_CACHE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int N = NQ * S2_R * B;
    const bool cached = B * NQ <= S2_LAYOUT_CACHE;
    if (cached)
        for (int x = tid; x < B * NQ; x += 1024) gcache[x] = groups[x];
    __syncthreads();
    auto group_of = [&](int b, int q) { return cached ? gcache[b * NQ + q] : groups[(size_t)b * NQ + q]; };
    auto count = [&](int b, int q, int sub) {
        const int hq = min(S2_R, L - q * S2_R);
        const int grp = group_of(b, q);
        // the first strip starts at t = 0 and has no ghost columns
        if (grp >= 0)
            return sub != 0 ? 0 : P <= wcap ? 1 : 1 + (P - wcap + (wcap - grp) - 1) / (wcap - grp);
        return sub < hq ? (P + wcap - 1) / wcap : 0;
    };
    int base = 0;                                   // tickets before this tile
    for (int e0 = 0, it = 0; e0 < N; e0 += 1024, ++it) {
        const int e = e0 + tid;
        int c = 0, prev = -1, prev_cnt = 0, g = -1;
        if (e < N) {
            const int level = e / B, b = e - level * B;
            const int q = level / S2_R, sub = level % S2_R;
            c = count(b, q, sub);
            const int grp = group_of(b, q);
            g = grp >= 0 && sub == 0 ? grp : -1;
            if (sub > 0) {
                prev = e - B;
                prev_cnt = count(b, q, sub - 1);
            } else if (q > 0) {
                const int psub = group_of(b, q - 1) >= 0 ? 0 : S2_R - 1;
                prev = ((q - 1) * S2_R + psub) * B + b;
                prev_cnt = count(b, q - 1, psub);
            }
        }
        // inclusive scan of c inside the wave
        int incl = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int v = __shfl_up(incl, d, 64);
            if (lane >= d) incl += v;
        }
        if (lane == 63) wsum[it & 1][wave] = incl;
        __syncthreads();
        int before = 0, tile_total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int v = wsum[it & 1][w];
            if (w < wave) before += v;
            tile_total += v;
        }
        const int tstart = base + before + incl - c;
        if (e < N) {
            S2Entry en;
            en.cnt = c;
            en.prev = prev;
            en.prev_cnt = prev_cnt;
            en.g = g;
            entries[e] = en;
            for (int x = 0; x < c; ++x) {
                S2Task t;
                t.entry = e;
                t.strip = x;
                tasks[tstart + x] = t;
            }
        }
        base += tile_total;
    }
    if (tid == 0) hdr->total = (uint32_t)base;
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

// M and K travel between workgroups on different compute units (and L2
// slices): they are written with agent-scope stores, which go through to the
// level every compute unit sees, and read back with agent-scope loads, which
// do not use a copy cached before the write.  A task counts as complete once
// the vector-memory counter of every wave has drained (the stores have been
// acknowledged) and the completion counter has then been incremented.
__device__ __forceinline__ void st_agent(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint8_t* p, uint8_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Workgroup barrier that orders LDS accesses only.  The vector-memory counter
// is left alone, so global -> LDS copies for later chunks stay in flight
// across it; the copies a barrier must cover are waited for explicitly
// (wait_vm) before it.
// (Written as assembly because the compiler otherwise drains every counter in
// front of a barrier instruction.)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
constexpr int DMA_AGENT_SCOPE = 16;        // cache-policy bit sc1 of the global -> LDS load

// Wait until at most `later` of the vector-memory operations this wave has
// issued are still outstanding.  They complete in order, so this waits for
// everything issued before the last `later` ones.  A smaller number only waits
// longer, so the count is clamped to what the instruction can encode here.
__device__ __forceinline__ void wait_vm(int later)
{
    // s_waitcnt immediates: vmcnt in bits 3:0 (and 15:14), expcnt 6:4 and lgkmcnt 11:8 left alone
    switch (later) {
        case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
        case 1: __builtin_amdgcn_s_waitcnt(0x0F71); break;
        case 2: __builtin_amdgcn_s_waitcnt(0x0F72); break;
        case 3: __builtin_amdgcn_s_waitcnt(0x0F73); break;
        case 4: __builtin_amdgcn_s_waitcnt(0x0F74); break;
        case 5: __builtin_amdgcn_s_waitcnt(0x0F75); break;
        case 6: __builtin_amdgcn_s_waitcnt(0x0F76); break;
        case 7: __builtin_amdgcn_s_waitcnt(0x0F77); break;
        default: __builtin_amdgcn_s_waitcnt(0x0F78); break;
    }
}

// Copy the part x in [x0, x0 + 256*NGK) of the window tp in [lo, lo + n) of a
// row of M into slot[0..n): -inf for tp < 0, nothing for tp >= tlimit.  Run by
// one wave; the window is cut into 16-byte groups, one per lane and pass.  A
// group inside [0, tlimit) goes global -> LDS without passing registers (the
// lanes fill consecutive 16-byte cells from a wave-uniform LDS base); a group
// entirely below 0 is one 16-byte store of -inf; the at most two groups that
// straddle 0 or tlimit are written element by element.  `row0`: the row is the
// base case M[0][t] = +0, not read from memory.  Returns the number of
// global -> LDS loads issued with at least one lane.
template <int NGK>
__device__ __forceinline__ int stage_window(float* slot, const float* row, int lo, int n,
                                            int tlimit, bool row0, int x0, int lane)
{
    constexpr float NINF = -INFINITY;
    int issued = 0;
    if (!row0 && lo >= 0 && lo + ((n + 3) & ~3) <= tlimit) {
        // the common case: every group is inside the row
#pragma unroll
        for (int k = 0; k < NGK; ++k) {
            const int xb = x0 + 256 * k;           // wave-uniform
            const int x = xb + 4 * lane;
            if (xb < n) {
                ++issued;
                if (x < n)
                    __builtin_amdgcn_global_load_lds(row + lo + x, (lds_void*)(slot + xb), 16, 0,
                                                     DMA_AGENT_SCOPE);
            }
        }
        return issued;
    }
#pragma unroll
    for (int k = 0; k < NGK; ++k) {
        const int xb = x0 + 256 * k;
        const int x = xb + 4 * lane;
        const int tp = lo + x;
        const bool go = x < n && !row0 && tp >= 0 && tp + 3 < tlimit;
        if (__ballot(go) != 0) ++issued;
        if (x < n) {
            if (go) {
                __builtin_amdgcn_global_load_lds(row + tp, (lds_void*)(slot + xb), 16, 0,
                                                 DMA_AGENT_SCOPE);
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
                        if (tpe >= 0) v = row0 ? 0.0f : ld_agent(row + tpe);
                        slot[x + e] = v;
                    }
                }
            }
        }
    }
    return issued;
}

template <int NT, int U, int CH, int DMAX, int WPE, int NBUF, bool STORE_K>
__global__ __launch_bounds__(NT, WPE) void stage2_tiled_kernel(
    int B, int L, int P, float* M, uint8_t* K, S2Header* hdr, uint32_t* done,
    const S2Entry* __restrict__ entries, const S2Task* __restrict__ tasks,
    const S2Rec* __restrict__ recs, const S2Info* __restrict__ infos,
    const S2Shift* __restrict__ shifts, int NQ, long long wait_limit)
{
    constexpr int R = S2_R;
    constexpr int WCAP = NT * U;
    constexpr int SLOTW = WCAP + DMAX + 4;  // multiple of 4
    constexpr float NINF = -INFINITY;
    static_assert(2 * CH >= R - 1, "the diagonal part needs R-1 slots");
    __shared__ __attribute__((aligned(16))) float bufA[CH][SLOTW];
    __shared__ __attribute__((aligned(16))) float bufB[CH][SLOTW];
    static_assert(NBUF == 2 || NBUF == 3, "two or three window buffers");
    __shared__ __attribute__((aligned(16))) float bufC[NBUF == 3 ? CH : 1][NBUF == 3 ? SLOTW : 4];
    __shared__ int sh_word[4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ld = L + 1;
    // columns: a wave owns U*64 consecutive columns, lane + 64*u inside them
    const int tl0 = wave * (64 * U) + lane;
    // window copies: WPR waves share a row of a chunk, each a run of 16-byte groups
    constexpr int NW = NT / 64;
    static_assert(NW % CH == 0, "waves must divide evenly over the rows of a chunk");
    constexpr int WPR = NW / CH;
    constexpr int NGK = (SLOTW / 4 + WPR * 64 - 1) / (WPR * 64);   // passes per wave
    const int st_row = wave / WPR;                  // row of the chunk this wave copies
    const int st_x0 = (wave - st_row * WPR) * (256 * NGK);

    const int total = (int)hdr->total;
#ifdef DPC_S2_TIMERS
    long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const long long tkernel0 = wall_clock64();
#endif
    for (;;) {
        TMARK(t_a);
        // ---- next ticket, its task, and the wait for the previous level of the
        //      instance (all by one lane; the rest of the workgroup waits at the barrier)
        if (tid == 0) {
            const int ticket = (int)atomicAdd(&hdr->ticket, 1u);
            int e = -1, strip = 0, g = -1, ok = 1;
            if (ticket < total) {
                const S2Task tk = tasks[ticket];
                const S2Entry ent = entries[tk.entry];
                e = tk.entry;
                strip = tk.strip;
                g = ent.g;
                if (ent.prev >= 0) {
                    const uint32_t need = (uint32_t)ent.prev_cnt;
                    const uint32_t* flag = &done[ent.prev];
                    const long long start = wall_clock64();
                    while (ld_relaxed(flag) < need) {
                        if (ld_relaxed(&hdr->error) != 0) { ok = 0; break; }
                        if (wall_clock64() - start > wait_limit) {
                            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                            ok = 0;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
            }
            sh_word[0] = ok ? e : -1;
            sh_word[1] = strip;
            sh_word[2] = g;
        }
        __syncthreads();
        const int e = __builtin_amdgcn_readfirstlane(sh_word[0]);
        const int s = __builtin_amdgcn_readfirstlane(sh_word[1]);
        const int entg = __builtin_amdgcn_readfirstlane(sh_word[2]);
        __syncthreads();
#ifdef DPC_S2_TIMERS
        if (e < 0 && tid == 0) {
            tacc[7] = wall_clock64() - tkernel0;
            for (int q = 0; q < 8; ++q)
                atomicAdd((unsigned long long*)&hdr->pad[1 + 2 * q], (unsigned long long)tacc[q]);
            atomicAdd(&hdr->pad[21], 1u);
        }
#endif
        if (e < 0) return;                         // no ticket left, or a wait ran out: all leave
        const int level = e / B;
        const int b = e - level * B;
        const int q = level / R;
        const int sub = level - q * R;
        const bool full = entg >= 0;
        const int g = full && s > 0 ? entg : 0;    // the first strip has nothing to its left
        const int j0 = 1 + q * R;
        const int hq = min(R, ld - j0);
        const int rlo = full ? 0 : sub;            // rows of the group this task computes
        const int rhi = full ? hq : sub + 1;
        const int ilimit = j0 + rlo;               // rows below come from global memory
        const int weff = WCAP - g;
        const int t0 = s == 0 ? 0 : WCAP + (s - 1) * weff;   // first stored column
        const int tS = t0 - g;                     // first computed column
        const int tend = min(tS + WCAP, P);
        const int tstore_end = min(t0 + weff, P);
        float* Mb = M + (size_t)b * ld * P;
        uint8_t* Kb = STORE_K ? K + (size_t)b * ld * P : nullptr;
        const S2Rec* brec = recs + ((size_t)b * NQ + q) * ld;
        const S2Info* binfo = infos + ((size_t)b * NQ + q) * ld;
        const S2Shift* bshift = shifts + ((size_t)b * NQ + q) * ld;
        TMARK(t_b);
        TACC(3, t_a, t_b);

        // row 0, the base case, is written by the first level
        if (q == 0 && rlo == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tS + tl0 + 64 * u;
                if (t >= t0 && t < tstore_end) {
                    st_agent(Mb + t, 0.0f);
                    if (STORE_K) st_agent(Kb + t, (uint8_t)DPC_NOARG);
                }
            }
        }

        float best[R][U];
        int arg[R][U];
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int u = 0; u < U; ++u) { best[rr][u] = NINF; arg[rr][u] = DPC_NOARG; }

        // a one-row task uses only row `sub` of a predecessor: its shift (-1: no
        // candidate) and importance
        auto one_row_of = [&](int i, int& w, float& imp) __attribute__((always_inline)) {
            const S2Shift sh = bshift[i];
            const S2Rec rec = brec[i];
            w = -1;
            imp = NINF;
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
                if (rr == sub) { w = sh.w[rr]; imp = rec.imp[rr]; }
        };

        // a wave whose columns all lie beyond the table has nothing to relax
        const bool wave_idle = tS + wave * (64 * U) >= tend;

        // start the copy of this wave's part of the window of row i0 + st_row
        // into `buf` (asynchronous); returns the number of loads issued
        auto stage_chunk = [&](float (*buf)[SLOTW], int i0) __attribute__((always_inline)) {
            const int i = i0 + st_row;
            if (i >= ilimit) return 0;
            S2Info inf = binfo[i];
            if (!full) {
                int w;
                float imp;
                one_row_of(i, w, imp);
                inf.mins = inf.maxs = w;
            }
            // (a row none of whose shifts reaches the task is copied all the same:
            //  its window is then the -inf that lies below column 0)
            if (inf.maxs < 0) return 0;
            const int lo = tS - inf.maxs;
            const int n = tend - inf.mins - lo;
            if (st_x0 >= n) return 0;
            return stage_window<NGK>(buf[st_row], Mb + (size_t)i * P, lo, n, P, i == 0, st_x0,
                                     lane);
        };

        // relax the group's rows from the rows [i0, i0+CH) held in `buf`.
        // A candidate whose shift exceeds every column of the task reads the
        // part of the window that lies below column 0, which was filled with
        // -inf; a missing candidate adds -inf to whatever the slot holds: neither
        // needs a test here.
        auto relax_chunk = [&](const float (*buf)[SLOTW], int i0, const S2Rec (&rec)[CH])
                               __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int i = i0 + c;
                if (i >= ilimit) continue;
                const char* base = (const char*)&buf[c][tl0];
                // LDS reads run one row of the group ahead of the arithmetic
                float mcur[U], mnxt[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    mcur[u] = *(const float*)(base + rec_off4(rec[c], 0) + 256 * u);
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    if (rr + 1 < R) {
#pragma unroll
                        for (int u = 0; u < U; ++u)
                            mnxt[u] = *(const float*)(base + rec_off4(rec[c], rr + 1) + 256 * u);
                    }
                    const float imp = rec[c].imp[rr];
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
            }
        };

        // One chunk step: fetch the chunk's records (one batch of scalar loads,
        // in flight across the barrier), wait for this chunk's window copies
        // (the copies of the next chunk, `later` instructions, may stay in
        // flight), start the copies of the chunk two ahead into the buffer that
        // was relaxed last, relax.
        int later = 0;         // copies in flight for the chunk after the current one
        // (A one-row task has its own, simple relax so that the whole-group path
        //  keeps its records untouched in scalar registers.)
        auto relax_one_row = [&](const float (*buf)[SLOTW], int i0) __attribute__((always_inline)) {
            for (int c = 0; c < CH; ++c) {
                const int i = i0 + c;
                if (i >= ilimit) break;
                int w;
                float imp;
                one_row_of(i, w, imp);
                if (w < 0) continue;
                const float* base = &buf[c][tl0];       // the window starts at tS - w
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    if (rr != sub) continue;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const float cand = base[64 * u] + imp;
                        if (cand > best[rr][u]) { best[rr][u] = cand; arg[rr][u] = i; }
                    }
                }
            }
        };
        auto chunk_step = [&](auto whole, float (*cur)[SLOTW], float (*free2)[SLOTW], int i0)
                              __attribute__((always_inline)) {
            constexpr bool WHOLE = decltype(whole)::value;
            S2Rec rec[CH];
            if (WHOLE && !wave_idle) {
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const S2Rec* r = &brec[min(i0 + c, L)];
#pragma unroll
                    for (int x = 0; x < R / 2; ++x) rec[c].offp[x] = r->offp[x];
#pragma unroll
                    for (int x = 0; x < R; ++x) rec[c].imp[x] = r->imp[x];
                }
            }
            TMARK(ta);
            wait_vm(later);
            lds_barrier();                             // `cur` filled, `free2` no longer read
            TMARK(tb);
            const int fresh = stage_chunk(free2, i0 + (NBUF - 1) * CH);
            TMARK(tc);
            if (!wave_idle) {
                if constexpr (WHOLE) relax_chunk(cur, i0, rec);
                else relax_one_row(cur, i0);
            }
            TMARK(td);
            TACC(0, ta, tb);
            TACC(1, tb, tc);
            TACC(2, tc, td);
            return fresh;
        };
        auto off_diagonal = [&](auto whole) __attribute__((always_inline)) {
            // (the barrier that ended the previous task has freed all buffers)
            stage_chunk(bufA, 0);
            if constexpr (NBUF == 3) {
                later = stage_chunk(bufB, CH);
                for (int i0 = 0; i0 < ilimit; i0 += 3 * CH) {
                    later = chunk_step(whole, bufA, (float (*)[SLOTW])bufC, i0);
                    if (i0 + CH < ilimit) later = chunk_step(whole, bufB, bufA, i0 + CH);
                    if (i0 + 2 * CH < ilimit)
                        later = chunk_step(whole, (float (*)[SLOTW])bufC, bufB, i0 + 2 * CH);
                }
            } else {
                // two buffers: the copy in flight is always the one waited for next
                for (int i0 = 0; i0 < ilimit; i0 += 2 * CH) {
                    chunk_step(whole, bufA, bufB, i0);
                    later = 0;
                    if (i0 + CH < ilimit) chunk_step(whole, bufB, bufA, i0 + CH);
                    later = 0;
                }
            }
        };

        // ---------------- off-diagonal part: rows i < ilimit ----------------
        if (full) off_diagonal(std::true_type{});
        else off_diagonal(std::false_type{});
        TMARK(t_c);
        __syncthreads();                               // off-diagonal readers done
        if (full && tS == 0) {
            // first strip: what lies to the left of column 0 does not exist
            for (int x = tid; x < (R - 1) * DMAX; x += NT) {
                const int rr = x / DMAX;
                float* slot = rr < CH ? bufA[rr] : bufB[rr - CH];
                slot[x - rr * DMAX] = NINF;
            }
        }

        // ---------------- diagonal part and output ----------------
        // records of the group's own rows, fetched four at a time
        S2Rec drec[4];
        int dmaxs[4];
        auto load_diag = [&](int first) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                drec[c] = brec[min(j0 + first + c, L)];
                dmaxs[c] = binfo[min(j0 + first + c, L)].maxs;
            }
        };
        if (full && !wave_idle) load_diag(0);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int j = j0 + rr;
            if (rr >= rlo && rr < rhi) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = tS + tl0 + 64 * u;
                    if (t >= t0 && t < tstore_end) {
                        st_agent(Mb + (size_t)j * P + t, best[rr][u]);
                        if (STORE_K) st_agent(Kb + (size_t)j * P + t, (uint8_t)arg[rr][u]);
                    }
                }
            }
            if (rr + 1 < R) {
                // row j of a whole-group task feeds the rows below it through an LDS
                // slot: own column t at slot position DMAX + (t - tS)
                const bool feeds = full && rr + 1 < rhi;
                float* slot = rr < CH ? bufA[rr] : bufB[rr - CH];
                if (feeds) {
#pragma unroll
                    for (int u = 0; u < U; ++u) slot[DMAX + tl0 + 64 * u] = best[rr][u];
                }
                __syncthreads();
                if (feeds && !wave_idle) {
                    const S2Rec& rec = drec[rr & 3];
                    const int maxs = dmaxs[rr & 3];
                    if (maxs >= 0) {
#pragma unroll
                        for (int r2 = rr + 1; r2 < R; ++r2) {
                            // shifts inside a group are at most DMAX: a shift beyond
                            // the task's last column can only occur in the first
                            // strip, whose pad holds -inf
                            const int w = maxs - (rec_off4(rec, r2) >> 2);
                            const float imp = rec.imp[r2];
                            const float* sp = &slot[DMAX - w + tl0];
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const float cand = sp[64 * u] + imp;
                                if (cand > best[r2][u]) { best[r2][u] = cand; arg[r2][u] = j; }
                            }
                        }
                    }
                    if (rr == 3) load_diag(4);
                }
            }
        }
        TMARK(t_d);
        TACC(4, t_c, t_d);

        // ---- publish: one more task of this entry is complete
        wait_vm(0);                                    // this wave's stores are acknowledged
        __syncthreads();                               // ... every wave's; also frees the buffers
        if (tid == 0)
            __hip_atomic_fetch_add(&done[e], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        TMARK(t_e);
        TACC(5, t_d, t_e);
    }
}

template <int NT, int U, int CH, int DMAX, int WPE, int NBUF>
static hipError_t launch_cfg(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                             uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    constexpr int WCAP = NT * U;
    const int NQ = (L + S2_R - 1) / S2_R;
    const S2Layout lay = s2_layout(B, L, P);
    if (lay.nentries > 0x3FFFFFF0LL || lay.maxtasks > 0x3FFFFFF0LL) return hipErrorInvalidValue;
    const int N = (int)lay.nentries;
    char* base = (char*)workspace;
    S2Header* hdr = (S2Header*)base;
    uint32_t* done = (uint32_t*)(base + lay.done_off);
    S2Entry* entries = (S2Entry*)(base + lay.entry_off);
    S2Task* tasks = (S2Task*)(base + lay.task_off);
    int32_t* groups = (int32_t*)(base + lay.group_off);
    S2Rec* recs = (S2Rec*)(base + lay.rec_off);
    S2Info* infos = (S2Info*)(base + lay.info_off);
    S2Shift* shifts = (S2Shift*)(base + lay.shift_off);

    hipError_t e = launch_clear_words(workspace, (int)(sizeof(S2Header) / 4) + N, st);
    if (e != hipSuccess) return e;
    // ghost columns cost recomputation: at most a quarter of a task, and the
    // chain of shifts must fit the pad in front of a diagonal slot
    const int gmax = std::min(DMAX, WCAP / 4);
    hipLaunchKernelGGL(stage2_pack_kernel, dim3(NQ, B), dim3(256), 0, st, L, P, NQ, Topt, I, recs,
                       infos, shifts, groups, gmax, DMAX, WCAP);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stage2_layout_kernel, dim3(1), dim3(1024), 0, st, B, L, P, NQ, WCAP, groups,
                       entries, tasks, hdr);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    // resident workgroups per compute unit: WPE waves per SIMD, 4 SIMDs
    constexpr int wg_per_cu = (WPE * 4 * 64) / NT;
    static_assert(wg_per_cu >= 1, "a workgroup must fit one compute unit");
    const int grid = num_cu * wg_per_cu;
    const long long wait_limit = 500000000LL;      // 5 s of the 100 MHz wall clock
    if (K)
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, WPE, NBUF, true>), dim3(grid), dim3(NT),
                           0, st, B, L, P, M, K, hdr, done, entries, tasks, recs, infos, shifts,
                           NQ, wait_limit);
    else
        hipLaunchKernelGGL((stage2_tiled_kernel<NT, U, CH, DMAX, WPE, NBUF, false>), dim3(grid),
                           dim3(NT), 0, st, B, L, P, M, K, hdr, done, entries, tasks, recs, infos,
                           shifts, NQ, wait_limit);
    return hipGetLastError();
}

int g_s2_shape = 0;     // tuning override, see launch_stage2_tiled

hipError_t launch_stage2_tiled(int B, int L, int P, const int32_t* Topt, const float* I, float* M,
                               uint8_t* K, void* workspace, int num_cu, hipStream_t st)
{
    // WCAP = NT*U columns per task.  Narrow tables take the narrowest shape that
    // covers them.  Wide tables use 1024 columns per task: with many rows (long
    // tasks) two workgroups per compute unit and three window buffers, with few
    // rows (short tasks, latency-bound) three workgroups and two buffers
    // (measured on the stress, L=100 and L=53 workloads).
    int shape = g_s2_shape;
    if (shape == 0) {
        if (P <= 256) shape = 1;
        else if (P <= 512) shape = 2;
        else shape = L >= 128 ? 4 : 6;
    }
    switch (shape) {
        case 1: return launch_cfg<256, 1, 4, 240, 4, 3>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 2: return launch_cfg<256, 2, 4, 240, 4, 3>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 3: return launch_cfg<256, 4, 4, 240, 4, 2>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 4: return launch_cfg<512, 2, 4, 256, 4, 3>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 5: return launch_cfg<1024, 2, 4, 256, 4, 3>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        case 6: return launch_cfg<512, 2, 4, 256, 6, 2>(B, L, P, Topt, I, M, K, workspace, num_cu, st);
        default: return hipErrorInvalidValue;
    }
}

int stage2_tiled_error(const void* workspace_host_copy)
{
    return (int)((const S2Header*)workspace_host_copy)->error;
}

}  // namespace dpc
