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
// load; a second small kernel lays out the task table and the first also
// writes row 0 of M, the base case (see stage2_pack.hip).
#include "stage2_common.h"

namespace dpc {

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
        const int j0 = s2_group_first_row(L, R, q);
        const int hq = s2_group_rows(L, R, q);     // rows of the group; the other row slots are empty
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
    const S2Layout lay = s2_layout(B, L, P, S2_R);
    if (lay.nentries > 0x3FFFFFF0LL || lay.maxtasks > 0x3FFFFFF0LL) return hipErrorInvalidValue;
    char* base = (char*)workspace;
    S2Header* hdr = (S2Header*)base;
    uint32_t* done = (uint32_t*)(base + lay.done_off);
    S2Entry* entries = (S2Entry*)(base + lay.entry_off);
    S2Task* tasks = (S2Task*)(base + lay.task_off);
    S2Rec* recs = (S2Rec*)(base + lay.rec_off);
    S2Info* infos = (S2Info*)(base + lay.info_off);
    S2Shift* shifts = (S2Shift*)(base + lay.shift_off);

    // ghost columns cost recomputation: at most a quarter of a task, and the
    // chain of shifts must fit the pad in front of a diagonal slot
    const int gmax = std::min(DMAX, WCAP / 4);
    hipError_t e = launch_stage2_prepare(B, L, P, S2_R, Topt, I, M, K, workspace, gmax, DMAX, DMAX, WCAP, 0, st);
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