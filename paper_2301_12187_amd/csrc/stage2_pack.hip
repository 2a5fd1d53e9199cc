// Preparation kernels of the persistent stage-2 family: workspace layout,
// operand records (Topt and I repacked per row group), task table.
#include "stage2_common.h"

namespace dpc {

S2Layout s2_layout(int B, int L, int P, int R)
{
    S2Layout l;
    const size_t nq = ((size_t)L + R - 1) / R;
    const size_t halves = (size_t)R / S2_H;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    l.nentries = (long long)nq * R * B;
    // most tasks arise when every group runs row by row with the narrowest strips
    l.maxtasks = l.nentries * (((long long)P + 255) / 256);
    l.done_off = sizeof(S2Header);
    l.entry_off = up(l.done_off + 4 * (size_t)l.nentries);
    l.group_off = up(l.entry_off + sizeof(S2Entry) * ((size_t)l.nentries + 1));
    l.task_off = up(l.group_off + 4 * (size_t)B * nq);
    l.rec_off = up(l.task_off + sizeof(S2Task) * (size_t)l.maxtasks);
    l.info_off = up(l.rec_off + sizeof(S2Rec) * halves * B * nq * (L + 1));
    l.shift_off = up(l.info_off + sizeof(S2Info) * (size_t)B * nq * (L + 1));
    l.total = up(l.shift_off + sizeof(S2Shift) * halves * B * nq * (L + 1));
    return l;
}

// (the caller sizes the workspace before a kernel family is chosen)
size_t stage2_workspace_bytes(int B, int L, int P)
{
    return std::max(s2_layout(B, L, P, 8).total, s2_layout(B, L, P, 16).total);
}

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
// row i offers to the rows j0..j0+hq-1 of the group (R row slots), stored as
// R/8 consecutive S2Rec of eight rows each.  A candidate exists when i < j,
// j is a row of the group and 0 <= Topt[i][j] < P.  Shifts are stored as offsets below the
// largest shift of the record, the position of the candidate inside the LDS
// window of row i; a missing candidate has importance -inf and so never wins
// whatever it is added to.  The workgroups of the first group also write row
// 0 of M (and K).  The workgroup also decides how the group runs:
// groups[b][q] = (ghost width g, largest spread) if every spread fits dspread,
// every shift inside the group fits dpad and g <= gmax, else -1 (row by row).
template <int R>
__global__ __launch_bounds__(256) void stage2_pack_kernel(
    int L, int P, int NQ, ToptRef Topt, const float* __restrict__ I,
    S2Rec* __restrict__ recs, S2Info* __restrict__ infos, S2Shift* __restrict__ shifts,
    int32_t* __restrict__ groups, int gmax, int dspread, int dpad, int wcap, int ahead, int ringf,
    float* __restrict__ M, uint8_t* __restrict__ K, S2Gate gate, uint32_t* __restrict__ hdr_words,
    uint32_t* __restrict__ done, int keep_word)
{
    if (s2_gate_closed(gate)) return;
    constexpr int H = R / S2_H;            // records per (group, predecessor)
    // What the main kernel expects to find zero: the completion counters of the
    // R levels of this (group, instance), and, from the first workgroup, the
    // header (ticket, error; the layout kernel fills in the rest afterwards).
    // keep_word >= 0: a header word that is left alone (the choice a gated
    // preparation was made conditional on).
    if (threadIdx.x < R)
        done[((size_t)blockIdx.x * R + threadIdx.x) * gridDim.y + blockIdx.y] = 0;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < sizeof(S2Header) / 4 &&
        (int)threadIdx.x != keep_word)
        hdr_words[threadIdx.x] = 0;
    __shared__ int wd[R][R];
    // dynamic LDS, sized by the launch for nt = blockDim.x threads: the columns of
    // Topt and I that the group reads, nt rows of R + 1 words each, then the
    // window bounds of every predecessor
#ifndef DPC_HOST_EMU
    extern __shared__ __attribute__((aligned(16))) char pack_lds[];
#else
    char* const pack_lds = emu::g_dyn_lds;
#endif
    const int nt = (int)blockDim.x;
    int32_t (*sT)[R + 1] = (int32_t (*)[R + 1])pack_lds;
    float (*sI)[R + 1] = (float (*)[R + 1])(pack_lds + (size_t)nt * (R + 1) * 4);
    int* const smax = (int*)(pack_lds + (size_t)nt * (R + 1) * 8);
    int* const smin = smax + nt;
    __shared__ int spread;                 // largest spread of a predecessor's shifts into the group
    __shared__ int row_by_row;             // the group does not fit a whole-group task
    const int ld = L + 1;
    const int i = threadIdx.x;             // one thread per predecessor (L + 1 of them, whole waves)
    const int q = blockIdx.x;
    const int b = blockIdx.y;
    const int j0 = s2_group_first_row(L, R, q);
    const int hq = s2_group_rows(L, R, q);
    if (i == 0) spread = 0;
    __syncthreads();
    if (q == 0) {
        // the base case of the recurrence: M[0][t] = +0 for every budget, no arg-max
        float* M0 = M + (size_t)b * ld * P;
        for (int t = i; t < P; t += nt) M0[t] = 0.0f;
        if (K) {
            uint8_t* K0 = K + (size_t)b * ld * P;
            for (int t = i; t < P; t += nt) K0[t] = (uint8_t)DPC_NOARG;
        }
    }
    // the R columns j0 .. j0+R-1 of Topt and I, staged through LDS so that the
    // loads run along the rows (R consecutive words per row)
    // (nt >= L + 1, so R passes cover the L + 1 rows; the loads of all passes are
    //  issued before the first is used)
    int32_t tv[R];
    float iv[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int x = i + k * nt;
        const int row = x / R, rr = x - row * R;
        const bool ok = row < ld && rr < hq;
        tv[k] = 0;
        iv[k] = 0.0f;
        if (ok) Topt.operands(I, b, ld, row, j0 + rr, tv[k], iv[k]);
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int x = i + k * nt;
        const int row = x / R, rr = x - row * R;
        if (row < ld && rr < hq) {
            sT[row][rr] = tv[k];
            sI[row][rr] = iv[k];
        }
    }
    __syncthreads();
    S2Rec rec[H];
    int wv[R];
    int mins = 0x7FFFFFFF, maxs = -1;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int j = j0 + rr;
        int w = -1;
        float imp = -INFINITY;
        if (i < ld && rr < hq && i < j) {
            const int v = sT[i][rr];
            if (v >= 0 && v < P) {
                w = v;
                imp = sI[i][rr];
                mins = min(mins, w);
                maxs = max(maxs, w);
            }
        }
        wv[rr] = w;
        rec[rr / S2_H].imp[rr % S2_H] = imp;
    }
#pragma unroll
    for (int rr = 0; rr < R / 2; ++rr) {
        // a spread beyond dmax sends the group to the row-by-row path, which does
        // not use these offsets: clamp so that the halves cannot overflow
        const uint32_t lo = wv[2 * rr] < 0 ? 0u : (uint32_t)min(maxs - wv[2 * rr], 16383) * 4u;
        const uint32_t hi = wv[2 * rr + 1] < 0 ? 0u : (uint32_t)min(maxs - wv[2 * rr + 1], 16383) * 4u;
        rec[rr / (S2_H / 2)].offp[rr % (S2_H / 2)] = lo | (hi << 16);
    }
    // the window of row i that the group needs (none: any window will do),
    // and that of the row `ahead` rows further on, whose copy a kernel starts
    // while it works on row i
    smax[i] = max(maxs, 0);
    smin[i] = maxs < 0 ? 0 : mins;
    if (i < j0 && maxs >= 0) atomicMax(&spread, maxs - mins);
    __syncthreads();
    // ahead < 0: the kernel sizes its ring slots by the group's spread and
    // works -ahead rows ahead at most, fewer when the slots are large
    const int ahead_q = ahead >= 0 ? ahead : min(-ahead, s2_rows_ahead(ringf, spread));
#pragma unroll
    for (int h = 0; h < H; ++h) {
        rec[h].pad[0] = (uint32_t)smax[i];
        rec[h].pad[1] = i + ahead_q < ld ? (uint32_t)smax[i + ahead_q] : 0u;
        rec[h].pad[2] = i + ahead_q < ld ? (uint32_t)smin[i + ahead_q] : 0u;
        rec[h].pad[3] = (uint32_t)i;
    }
    // (rows above the group offer it nothing and their records are never read)
    const bool mine = i < ld && i < j0 + R;
    const size_t idx = ((size_t)b * NQ + q) * ld + i;
    if (mine) {
#pragma unroll
        for (int h = 0; h < H; ++h) recs[idx * H + h] = rec[h];
        infos[idx].mins = mins;
        infos[idx].maxs = maxs;
    }
    if (i >= j0 && i < j0 + R) {             // (slots past the group's rows offer nothing)
#pragma unroll
        for (int rr = 0; rr < R; ++rr) wd[i - j0][rr] = i < j0 + hq ? wv[rr] : -1;
    }
    __syncthreads();
    if (i == 0) {
        // how far to the left of its stored columns each row must be correct
        int need[R];
        int g = 0, hmax = 0;
#pragma unroll
        for (int rr = R - 1; rr >= 0; --rr) {
            int n = 0;
#pragma unroll
            for (int r2 = rr + 1; r2 < R; ++r2)
                if (wd[rr][r2] >= 0) {
                    n = max(n, wd[rr][r2] + need[r2]);
                    hmax = max(hmax, wd[rr][r2]);
                }
            need[rr] = n;
            g = max(g, n);
        }
        // a table that fits one task has no strip to its left: no ghost columns
        const bool bad = spread > dspread || hmax > dpad || (P > wcap && g > gmax);
        groups[(size_t)b * NQ + q] = bad ? -1 : s2_group_code(g, spread);
        row_by_row = bad ? 1 : 0;
    }
    __syncthreads();
    // the shifts themselves are read by the row-by-row path only
    if (row_by_row && mine) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) shifts[idx * H + rr / S2_H].w[rr % S2_H] = wv[rr];
    }
}

// Task table: entries in ticket order (level-major, then instance), the task
// list (entry and strip of every ticket) and the total.  One workgroup per
// level.  It first counts the tickets of all lower levels (every thread sums
// the groups of some instances, then one reduction), then walks its own
// entries in tiles of 1024, one entry per thread (so that its stores are
// coalesced), with a running prefix sum of the strip counts: wave scan, then
// one combine of the 16 wave totals per tile.
__global__ __launch_bounds__(1024) void stage2_layout_kernel(
    int B, int L, int P, int NQ, int R, int wcap, const int32_t* __restrict__ groups,
    S2Entry* __restrict__ entries, S2Task* __restrict__ tasks, S2Header* hdr, S2Gate gate, bool decide)
{
    if (s2_gate_closed(gate)) return;
    __shared__ int wsum[2][16];
    __shared__ int red[16];
    __shared__ int redbad[16];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int level = blockIdx.x;                   // = q * R + sub
    const int q = level / R, sub = level % R;
    const int strips1 = (P + wcap - 1) / wcap;      // tasks of a one-row level
    auto group_of = [&](int b, int qq) { return groups[(size_t)b * NQ + qq]; };
    // tasks of a whole group with ghost width grp: the first strip starts at
    // t = 0 and has no ghost columns
    auto whole_count = [&](int code) {
        const int grp = s2_group_ghost(code);
        return P <= wcap ? 1 : 1 + (P - wcap + (wcap - grp) - 1) / (wcap - grp);
    };
    auto count = [&](int b, int qq, int ss) {
        const int hq = s2_group_rows(L, R, qq);
        const int grp = group_of(b, qq);
        if (grp >= 0) return ss != 0 ? 0 : whole_count(grp);
        return ss < hq ? strips1 : 0;
    };
    // the entry whose rows the entry (lev, b) needs last, its task count and
    // the first row it writes
    auto pred = [&](int lev, int b, int& prev, int& prev_cnt, int& prev_row0) {
        const int qq = lev / R, ss = lev % R;
        prev = -1;
        prev_cnt = 0;
        prev_row0 = -1;
        if (ss > 0) {
            prev = (lev - 1) * B + b;
            prev_cnt = count(b, qq, ss - 1);
            prev_row0 = s2_group_first_row(L, R, qq) + ss - 1;
        } else if (qq > 0) {
            const bool whole = group_of(b, qq - 1) >= 0;
            const int psub = whole ? 0 : s2_group_rows(L, R, qq - 1) - 1;   // its last level with tasks
            prev = ((qq - 1) * R + psub) * B + b;
            prev_cnt = count(b, qq - 1, psub);
            prev_row0 = s2_group_first_row(L, R, qq - 1) + psub;
        }
    };

    // ---- tickets before this level
    int part = 0, bad = 0;                          // bad: groups that run row by row
    for (int b = tid; b < B; b += 1024)
        for (int qq = 0; qq <= q; ++qq) {
            const int below = qq < q ? R : sub;     // levels of group qq that lie below this one
            if (below == 0) continue;
            const int grp = group_of(b, qq);
            part += grp >= 0 ? whole_count(grp) : strips1 * min(below, s2_group_rows(L, R, qq));
            bad += grp < 0 ? 1 : 0;
        }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        part += __shfl_xor(part, d, 64);
        bad += __shfl_xor(bad, d, 64);
    }
    if (lane == 0) { red[wave] = part; redbad[wave] = bad; }
    __syncthreads();
    int base = 0, allbad = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) { base += red[w]; allbad += redbad[w]; }

    // ---- this level's entries and tasks
    for (int b0 = 0, it = 0; b0 < B; b0 += 1024, ++it) {
        const int b = b0 + tid;
        const int e = level * B + b;
        int c = 0, g = -1, spread_q = 0;
        int prev = -1, prev_cnt = 0, prev_row0 = -1, prev2 = -1, prev2_cnt = 0, unused = -1;
        if (b < B) {
            c = count(b, q, sub);
            const int grp = group_of(b, q);
            g = grp >= 0 && sub == 0 ? s2_group_ghost(grp) : -1;
            spread_q = grp >= 0 && sub == 0 ? s2_group_spread(grp) : 0;
            pred(level, b, prev, prev_cnt, prev_row0);
            if (prev >= 0) pred(prev / B, b, prev2, prev2_cnt, unused);
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
        if (b < B) {
            S2Entry en;
            en.cnt = c;
            en.prev = prev;
            en.prev_cnt = prev_cnt;
            en.g = g;
            en.prev_row0 = prev_row0;
            en.prev2 = prev2;
            en.prev2_cnt = prev2_cnt;
            en.spread = spread_q;
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
    if (blockIdx.x == gridDim.x - 1) {
        if (tid == 0) hdr->total = (uint32_t)base;
        if (tid < 4) hdr->ninf[tid] = -INFINITY;
        // The workgroup of the last level has looked at every group (R >= 2: its
        // row is not the first of its group).  Where the caller has another shape
        // queued behind this one it sets the choice word: 1 (the other shape) if
        // more than 2 % of the groups run row by row (a group of 16 rows that does
        // costs about eight times a whole one, groups of 8 rows about a tenth
        // more overall), else 0.
        if (decide && tid == 0) hdr->choice = (long long)allbad * 50 > (long long)NQ * B ? 1u : 0u;
    }
}

hipError_t launch_stage2_prepare(int B, int L, int P, int R, ToptRef Topt, const float* I,
                                 float* M, uint8_t* K, void* workspace, int gmax, int dspread,
                                 int dpad, int wcap, int ahead, int ringf, hipStream_t st, bool gated,
                                 uint32_t want, bool decide)
{
    if (R != 8 && R != 16) return hipErrorInvalidValue;
    const int NQ = (L + R - 1) / R;
    const S2Layout lay = s2_layout(B, L, P, R);
    if (lay.nentries > 0x3FFFFFF0LL || lay.maxtasks > 0x3FFFFFF0LL) return hipErrorInvalidValue;
    char* base = (char*)workspace;
    S2Header* hdr = (S2Header*)base;
    const S2Gate gate{gated ? &hdr->choice : nullptr, want};
    S2Rec* recs = (S2Rec*)(base + lay.rec_off);
    S2Info* infos = (S2Info*)(base + lay.info_off);
    S2Shift* shifts = (S2Shift*)(base + lay.shift_off);
    int32_t* groups = (int32_t*)(base + lay.group_off);
    uint32_t* done = (uint32_t*)(base + lay.done_off);
    const int keep_word = gated ? (int)(offsetof(S2Header, choice) / 4) : -1;
    // one thread per predecessor, whole waves; LDS as laid out in the kernel
    const int nt = (L + 1 + 63) / 64 * 64;
    const size_t pack_lds = (size_t)nt * ((size_t)(R + 1) * 8 + 8);
    if (R == 8)
        hipLaunchKernelGGL(stage2_pack_kernel<8>, dim3(NQ, B), dim3(nt), pack_lds, st, L, P, NQ, Topt, I,
                           recs, infos, shifts, groups, gmax, dspread, dpad, wcap, ahead, ringf, M, K, gate,
                           (uint32_t*)hdr, done, keep_word);
    else
        hipLaunchKernelGGL(stage2_pack_kernel<16>, dim3(NQ, B), dim3(nt), pack_lds, st, L, P, NQ, Topt, I,
                           recs, infos, shifts, groups, gmax, dspread, dpad, wcap, ahead, ringf, M, K, gate,
                           (uint32_t*)hdr, done, keep_word);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stage2_layout_kernel, dim3(NQ * R), dim3(1024), 0, st, B, L, P, NQ, R, wcap,
                       (const int32_t*)groups, (S2Entry*)(base + lay.entry_off),
                       (S2Task*)(base + lay.task_off), hdr, gate, decide);
    return hipGetLastError();
}

}  // namespace dpc
