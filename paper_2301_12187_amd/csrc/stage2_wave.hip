// Stage 2, persistent family with wave-private windows (Algorithm 2 /
// recurrence Eq. 7 of the paper): M[j][t] = max_i fl32(M[i][t - Topt[i][j]] +
// I[i][j]), lowest arg-max.
//
// Tasks.  The rows 1..L of an instance are cut into groups of R = 8 or 16
// rows, the budget axis into strips of WCAP = NW*256 columns.  A task is
// (instance, row group, strip): it keeps the R x WCAP running (maximum,
// arg-max) pairs in registers, reads rows below its group from global memory
// and writes its own rows, so it carries no state from task to task.  Every row of M
// is read back once per group above it, and that traffic, not the arithmetic,
// bounds the kernel when tables are wide: hence the tall groups.  To fit 16
// rows x 4 columns per lane the arg-max indices are kept as bytes, four to a
// register, and updated in place with a sub-dword select.
//
// What differs is the off-diagonal part.  Every wave owns 64*U consecutive
// columns and feeds itself: for predecessor row i it copies the window of
// that row that ITS columns need, [tW - maxshift_i, tW + 64*U - minshift_i),
// into a slot of its own ring in LDS (global -> LDS loads, 16 bytes per lane,
// no registers), a few rows ahead of the row it is relaxing (the ring holds 5,
// 3 or 2 slots of a whole number of 128-float units, sized per task from the
// largest spread of shifts that the pack kernel found for the group).  Nothing in this
// part is shared between waves, so there is no workgroup barrier in it: a wave
// waits only for its own loads, with a counted wait that leaves the loads of
// the rows ahead in flight.  To make that count exact every row issues the
// same number of loads with every lane active and no branch around them:
//   - the window start is rounded down to a multiple of 4 columns, so a
//     16-byte cell lies entirely below column 0 or entirely at or above it;
//     cells below column 0 are fetched from sixteen bytes of -inf in the
//     workspace header (those cells mean "no (A, S) reaches this budget");
//   - cells past the part of the window that is needed are clamped to its
//     last cell (the lanes then ask for the same 16 bytes);
//   - the cell that straddles the end of the row reads up to three floats of
//     the next row, which exists because a predecessor row is never row L;
//     nothing that is stored depends on them.
// A row that offers no candidate to the group is fetched all the same; its
// importances are -inf in the records, so it never wins.
//
// Where the ring has five slots, the rows below the group are taken two at a
// time: a cell is offered the larger of the two rows' candidates (one
// three-way maximum with the running maximum), the byte that is kept is the
// number of the pair, and which of the two rows it was is settled once per cell
// when the last row below the group is done, by looking the even row's
// candidate up again (relax_pair_rows, PairCell, resolve_pairs).  Values and
// arg-max indices are those of the one-at-a-time update: the maximum of two
// candidates has the bits of whichever is larger, a strict comparison against
// the running maximum keeps the first pair that attains it, and inside the
// pair the lower row wins a tie.
//
// The diagonal part (predecessors inside the group) is shared by the waves of
// the workgroup: a finished row goes to one of two LDS
// slots (laid over the rings, which are idle by then) from which the rows
// below it are relaxed, one workgroup barrier per row.
#include "stage2_common.h"

namespace dpc {

// One relaxation of one cell: if cand > best then best = cand and byte BYTE of
// argp = vi (vi < 256), i.e. Eq. 7's max with the lowest arg-max kept when
// candidates arrive in ascending order.  The compare writes the lane mask that
// both selects read; the second select writes one byte of its destination and
// preserves the other three.  (Two wait states are required between a vector
// compare and a vector instruction that reads its mask.)
#ifndef DPC_HOST_EMU
#define DPC_RELAX_CELL(B)                                                                    \
    asm("v_cmp_gt_f32 vcc, %2, %0\n\t"                                                       \
        "s_nop 1\n\t"                                                                        \
        "v_cndmask_b32 %0, %0, %2, vcc\n\t"                                                  \
        "v_cndmask_b32_sdwa %1, %1, %3, vcc dst_sel:BYTE_" #B                                \
        " dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" #B " src1_sel:DWORD"                    \
        : "+v"(best), "+v"(argp)                                                             \
        : "v"(cand), "v"(vi)                                                                 \
        : "vcc")
#else  // the CPU emulation build of the tests spells the same update out
#define DPC_RELAX_CELL(B)                                                                    \
    do {                                                                                     \
        if (cand > best) {                                                                   \
            best = cand;                                                                     \
            argp = (argp & ~(0xFFu << (8 * B))) | ((vi & 0xFFu) << (8 * B));                 \
        }                                                                                    \
    } while (0)
#endif
// Without back-pointers (TRACK false) the update is the plain maximum: the
// table never holds -0 (row 0 is +0 and a sum is -0 only when both terms are),
// so the maximum has the bits of the first candidate that attains it, as the
// strict comparison would leave them.
template <int BYTE, bool TRACK>
__device__ __forceinline__ void relax_cell(float& best, uint32_t& argp, float cand, uint32_t vi)
{
    static_assert(BYTE >= 0 && BYTE < 4, "four arg-max bytes per register");
    if constexpr (!TRACK) {
#ifndef DPC_HOST_EMU
        // (the instruction itself: the library maximum would first re-quiet its operands)
        asm("v_max_f32 %0, %0, %1" : "+v"(best) : "v"(cand));
#else
        best = cand > best ? cand : best;
#endif
    }
    else if constexpr (BYTE == 0) DPC_RELAX_CELL(0);
    else if constexpr (BYTE == 1) DPC_RELAX_CELL(1);
    else if constexpr (BYTE == 2) DPC_RELAX_CELL(2);
    else DPC_RELAX_CELL(3);
}
#undef DPC_RELAX_CELL
// the larger of two candidates (never -0, never NaN: the bits of whichever is larger)
__device__ __forceinline__ float max_cand(float a, float b)
{
#ifndef DPC_HOST_EMU
    float m;
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(a), "v"(b));
    return m;
#else
    return b > a ? b : a;
#endif
}
// The pair step's update with back-pointers: the new maximum of a cell and two
// candidates is formed in the register of the first candidate (one three-way
// maximum), compared with the old one, and takes its place: 5 vector
// instructions per two candidates with the two additions.  The running maxima
// therefore move to another register at every step.  Where they live is fixed
// here rather than left to the register allocator (which otherwise spills one
// or two of them into the loop and copies dozens at its back edge): 17 slots of
// four registers, v60 .. v127.  A step of kind 0 takes the rows in ascending
// order, row r from slot r + 1 to slot r (slot 0 is free before it); a step of
// kind 1 takes them in descending order, row r from slot r back to slot r + 1.
// The loop over pairs alternates the two kinds, so the maxima are back in
// place at its back edge.
template <int STEP, int RR, int COL>
struct PairCell {
    static __device__ __forceinline__ void run(float& best, uint32_t& argp, float ca, float cb,
                                               uint32_t vc)
    {
        // (the plain form: the CPU emulation build, and any row the table below lacks)
        ca = cb > ca ? cb : ca;
        if (ca > best) {
            best = ca;
            argp = (argp & ~(0xFFu << (8 * COL))) | ((vc & 0xFFu) << (8 * COL));
        }
    }
};
#ifndef DPC_HOST_EMU
#define DPC_STR_(x) #x
#define DPC_STR(x) DPC_STR_(x)
#define DPC_BR(slot, col) DPC_BR_##slot##_##col
#define DPC_BR_0_0 60
#define DPC_BR_0_1 61
#define DPC_BR_0_2 62
#define DPC_BR_0_3 63
#define DPC_BR_1_0 64
#define DPC_BR_1_1 65
#define DPC_BR_1_2 66
#define DPC_BR_1_3 67
#define DPC_BR_2_0 68
#define DPC_BR_2_1 69
#define DPC_BR_2_2 70
#define DPC_BR_2_3 71
#define DPC_BR_3_0 72
#define DPC_BR_3_1 73
#define DPC_BR_3_2 74
#define DPC_BR_3_3 75
#define DPC_BR_4_0 76
#define DPC_BR_4_1 77
#define DPC_BR_4_2 78
#define DPC_BR_4_3 79
#define DPC_BR_5_0 80
#define DPC_BR_5_1 81
#define DPC_BR_5_2 82
#define DPC_BR_5_3 83
#define DPC_BR_6_0 84
#define DPC_BR_6_1 85
#define DPC_BR_6_2 86
#define DPC_BR_6_3 87
#define DPC_BR_7_0 88
#define DPC_BR_7_1 89
#define DPC_BR_7_2 90
#define DPC_BR_7_3 91
#define DPC_BR_8_0 92
#define DPC_BR_8_1 93
#define DPC_BR_8_2 94
#define DPC_BR_8_3 95
#define DPC_BR_9_0 96
#define DPC_BR_9_1 97
#define DPC_BR_9_2 98
#define DPC_BR_9_3 99
#define DPC_BR_10_0 100
#define DPC_BR_10_1 101
#define DPC_BR_10_2 102
#define DPC_BR_10_3 103
#define DPC_BR_11_0 104
#define DPC_BR_11_1 105
#define DPC_BR_11_2 106
#define DPC_BR_11_3 107
#define DPC_BR_12_0 108
#define DPC_BR_12_1 109
#define DPC_BR_12_2 110
#define DPC_BR_12_3 111
#define DPC_BR_13_0 112
#define DPC_BR_13_1 113
#define DPC_BR_13_2 114
#define DPC_BR_13_3 115
#define DPC_BR_14_0 116
#define DPC_BR_14_1 117
#define DPC_BR_14_2 118
#define DPC_BR_14_3 119
#define DPC_BR_15_0 120
#define DPC_BR_15_1 121
#define DPC_BR_15_2 122
#define DPC_BR_15_3 123
#define DPC_BR_16_0 124
#define DPC_BR_16_1 125
#define DPC_BR_16_2 126
#define DPC_BR_16_3 127
#define DPC_PAIR_CELL(STEP, RR, COL, IN, OUT)                                                \
    template <>                                                                              \
    struct PairCell<STEP, RR, COL> {                                                         \
        static __device__ __forceinline__ void run(float& best, uint32_t& argp, float ca,    \
                                                   float cb, uint32_t vc)                    \
        {                                                                                    \
            asm("v_max3_f32 %0, %2, %0, %3\n\t"                                              \
                "v_cmp_lt_f32 vcc, %2, %0\n\t"                                               \
                "s_nop 1\n\t"                                                                \
                "v_cndmask_b32_sdwa %1, %1, %4, vcc dst_sel:BYTE_" #COL                      \
                " dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" #COL " src1_sel:DWORD"          \
                : "+{v" DPC_STR(OUT) "}"(ca), "+v"(argp)                                     \
                : "{v" DPC_STR(IN) "}"(best), "v"(cb), "v"(vc)                               \
                : "vcc");                                                                    \
            best = ca;                                                                       \
        }                                                                                    \
    };
#define DPC_PAIR_ROW(r, r1)                                                                  \
    DPC_PAIR_CELL(0, r, 0, DPC_BR(r1, 0), DPC_BR(r, 0))                                      \
    DPC_PAIR_CELL(0, r, 1, DPC_BR(r1, 1), DPC_BR(r, 1))                                      \
    DPC_PAIR_CELL(0, r, 2, DPC_BR(r1, 2), DPC_BR(r, 2))                                      \
    DPC_PAIR_CELL(0, r, 3, DPC_BR(r1, 3), DPC_BR(r, 3))                                      \
    DPC_PAIR_CELL(1, r, 0, DPC_BR(r, 0), DPC_BR(r1, 0))                                      \
    DPC_PAIR_CELL(1, r, 1, DPC_BR(r, 1), DPC_BR(r1, 1))                                      \
    DPC_PAIR_CELL(1, r, 2, DPC_BR(r, 2), DPC_BR(r1, 2))                                      \
    DPC_PAIR_CELL(1, r, 3, DPC_BR(r, 3), DPC_BR(r1, 3))
DPC_PAIR_ROW(0, 1)
DPC_PAIR_ROW(1, 2)
DPC_PAIR_ROW(2, 3)
DPC_PAIR_ROW(3, 4)
DPC_PAIR_ROW(4, 5)
DPC_PAIR_ROW(5, 6)
DPC_PAIR_ROW(6, 7)
DPC_PAIR_ROW(7, 8)
DPC_PAIR_ROW(8, 9)
DPC_PAIR_ROW(9, 10)
DPC_PAIR_ROW(10, 11)
DPC_PAIR_ROW(11, 12)
DPC_PAIR_ROW(12, 13)
DPC_PAIR_ROW(13, 14)
DPC_PAIR_ROW(14, 15)
DPC_PAIR_ROW(15, 16)
#undef DPC_PAIR_ROW
#undef DPC_PAIR_CELL
#endif
// issue priority x mod 4 for this wave (the instruction takes an immediate)
__device__ __forceinline__ void rotate_priority(uint32_t x)
{
#ifndef DPC_HOST_EMU
    switch (x & 3u) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
    }
#else
    (void)x;
#endif
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in this order
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
// the running maximum against two candidates at once
__device__ __forceinline__ void max_cand2(float& best, float a, float b)
{
#ifndef DPC_HOST_EMU
    asm("v_max3_f32 %0, %0, %1, %2" : "+v"(best) : "v"(a), "v"(b));
#else
    best = a > best ? a : best;
    best = b > best ? b : best;
#endif
}

// global -> LDS copy of 16 bytes per lane, made by the lanes for which `active`
// holds (one instruction whatever the mask, as long as some lane is active):
// lane l writes dst + 16 l bytes
__device__ __forceinline__ void lds_load16_if(bool active, const float* src, float* dst)
{
#ifndef DPC_HOST_EMU
    if (active) __builtin_amdgcn_global_load_lds(src, (lds_void*)dst, 16, 0, DMA_AGENT_SCOPE);
#else
    emu::global_load_lds_if(active, src, dst, 16);
#endif
}

template <int R, int NW, int RINGF, int DMAX, int WPE, bool STORE_K>
__global__ __launch_bounds__(NW * 64, WPE) void stage2_wave_kernel(
    int B, int L, int P, float* M, uint8_t* K, S2Header* hdr, uint32_t* done,
    const S2Entry* __restrict__ entries, const S2Task* __restrict__ tasks,
    const S2Rec* __restrict__ recs, const S2Info* __restrict__ infos,
    const S2Shift* __restrict__ shifts, int NQ, long long wait_limit, S2Gate gate,
    ToptRef Topt, const float* __restrict__ I)
{
    if (s2_gate_closed(gate)) return;                // (another shape was chosen for this call)
    constexpr int U = 4;                             // columns per lane: one arg-max byte each
    constexpr int H = R / S2_H;                      // records per (group, predecessor)
    constexpr int NT = NW * 64;
    constexpr int WV = 64 * U;                       // columns per wave
    constexpr int WCAP = NW * WV;                    // columns per task
    // Per wave a ring of RINGF floats: a window holds WV + spread columns plus
    // 3 of alignment slack, in units of 128 floats; the ring has 5, 3 or 2
    // slots and the wave works 4, 2 or 1 rows ahead (chosen per task from the
    // spread the pack kernel found for the group).
    // DMAX: pad in front of a diagonal slot = largest shift inside a group.
    constexpr int DSLOTW = WCAP + DMAX + 4;          // floats per diagonal slot
    constexpr int LDSF = NW * RINGF > 2 * DSLOTW ? NW * RINGF : 2 * DSLOTW;
    constexpr float NINF = -INFINITY;
    // Two predecessors per step (relax_pair_rows).  With back-pointers the step
    // needs a table of the pairs' operands behind the diagonal slots for the
    // settlement (resolve_pairs): shapes whose LDS has no room for it take one
    // predecessor per step.  Without back-pointers only 16-row groups use it.
    constexpr int PAIR_TAB = 128 * R;                // entries: pairs below the group x rows
    constexpr bool PAIRS = STORE_K ? (LDSF - 2 * DSLOTW) * 4 >= PAIR_TAB * 8 : R == 16;
    static_assert(R == 8 || R == 16, "one or two records per predecessor");
    static_assert(RINGF >= 5 * 3 * S2W_UNIT, "five slots of the smallest window fit the ring");
    static_assert(WV == 256, "the window sizes in stage2_common.h are for 256 columns per wave");
    static_assert(DMAX % 4 == 0, "diagonal slots stay 16-byte aligned");
    __shared__ __attribute__((aligned(16))) float lds[LDSF];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ld = L + 1;
    const int tl0 = wave * WV + lane;                // column of the task, u = 0
    float* const ring = lds + wave * RINGF;
    const char* const lbase = (const char*)(ring + lane);
    const int tmaxg = (P - 1) & ~3;                  // last 16-byte cell that holds a column < P
    const float* const ninf = hdr->ninf;
    int* const sh_word = (int*)lds;                  // ticket broadcast (the rings are idle then)

    const int total = (int)hdr->total;
    int publish = -1;                              // entry of the task this workgroup just finished
    for (;;) {
        // ---- wave 0: count the finished task as complete, take the next ticket
        //      and look up its task.  All of it is wave-uniform code (one lane
        //      only issues the atomics and writes the result), so that the
        //      loop over tasks never diverges.
        if (wave == 0) {
            if (publish >= 0 && lane == 0)
                __hip_atomic_fetch_add(&done[publish], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int ticket = 0;
            if (lane == 0) ticket = (int)atomicAdd(&hdr->ticket, 1u);
            ticket = __builtin_amdgcn_readfirstlane(ticket);
            int e = -1, strip = 0, g = -1, ok = 1, prev = -1, prev_cnt = 0, prev_row0 = -1, spread = 0;
            if (ticket < total) {
                const S2Task tk = tasks[ticket];
                const S2Entry ent = entries[tk.entry];
                e = tk.entry;
                strip = tk.strip;
                g = ent.g;
                prev = ent.prev;
                prev_cnt = ent.prev_cnt;
                prev_row0 = ent.prev_row0;
                spread = ent.spread;
                // every row below prev_row0 is final once the entry before `prev`
                // is complete; `prev` itself is waited for when its rows come up
                if (ent.prev2 >= 0) {
                    const uint32_t need = (uint32_t)ent.prev2_cnt;
                    const uint32_t* flag = &done[ent.prev2];
                    const long long start = wall_clock64();
                    for (uint32_t spin = 0; ld_uniform(flag) < need; ++spin) {
                        // (the error word and the clock are looked at now and then only)
                        if ((spin & 15u) == 15u) {
                            if (ld_uniform(&hdr->error) != 0) { ok = 0; break; }
                            if (wall_clock64() - start > wait_limit) {
                                if (lane == 0)
                                    __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                                ok = 0;
                                break;
                            }
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
            }
            if (lane == 0) {
                sh_word[0] = ok ? e : -1;
                sh_word[1] = strip;
                sh_word[2] = g;
                sh_word[3] = prev;
                sh_word[4] = prev_cnt;
                sh_word[5] = prev_row0;
                sh_word[6] = spread;
            }
        }
        __syncthreads();
        const int e = __builtin_amdgcn_readfirstlane(sh_word[0]);
        const int s = __builtin_amdgcn_readfirstlane(sh_word[1]);
        const int entg = __builtin_amdgcn_readfirstlane(sh_word[2]);
        const int prev = __builtin_amdgcn_readfirstlane(sh_word[3]);
        const uint32_t prev_cnt = (uint32_t)__builtin_amdgcn_readfirstlane(sh_word[4]);
        const int prev_row0 = __builtin_amdgcn_readfirstlane(sh_word[5]);
        const int spread = __builtin_amdgcn_readfirstlane(sh_word[6]);
        __syncthreads();
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
        const int ilimit = j0 + rlo;               // rows below come from global memory
        const int weff = WCAP - g;
        const int t0 = s == 0 ? 0 : WCAP + (s - 1) * weff;   // first stored column
        const int tS = t0 - g;                     // first computed column
        const int tend = min(tS + WCAP, P);
        const int tstore_end = min(t0 + weff, P);
        const int tW = tS + wave * WV;             // first column of this wave
        float* Mb = M + (size_t)b * ld * P;
        uint8_t* Kb = STORE_K ? K + (size_t)b * ld * P : nullptr;
        const S2Rec* brec = recs + ((size_t)b * NQ + q) * ld * H;
        const S2Info* binfo = infos + ((size_t)b * NQ + q) * ld;
        const S2Shift* bshift = shifts + ((size_t)b * NQ + q) * ld * H;

        float best[R][U];
        uint32_t argp[R];                          // arg-max of column u in byte u
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
#pragma unroll
            for (int u = 0; u < U; ++u) best[rr][u] = NINF;
            argp[rr] = 0x01010101u * DPC_NOARG;
        }

        // a wave whose columns all lie beyond the table has nothing to do but
        // to take part in the barriers
        const bool wave_idle = tW >= tend;

        // Stores of a finished row: which of this lane's columns are stored and
        // at which offset from the start of the row does not depend on the row,
        // so a store is a wave-uniform row address plus a 32-bit lane offset.
        bool st_ok[U];
        unsigned st_off[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = tS + tl0 + 64 * u;               // >= 0: the first computed column is
            st_ok[u] = t >= t0 && t < tstore_end;
            st_off[u] = (unsigned)t;
        }
        auto store_row = [&](int j, int rr) __attribute__((always_inline)) {
            char* const mrow = (char*)(Mb + (size_t)j * P);
            uint8_t* const krow = STORE_K ? Kb + (size_t)j * P : nullptr;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (st_ok[u]) {
                    st_agent((float*)(mrow + 4u * st_off[u]), best[rr][u]);
                    if (STORE_K) st_agent(krow + st_off[u], (uint8_t)(argp[rr] >> (8 * u)));
                }
            }
        };

        // shift and importance of the candidate that row i offers to the row of
        // a one-row task (w = -1: none)
        auto one_row_of = [&](int i, int& w, float& imp) __attribute__((always_inline)) {
            w = -1;
            imp = NINF;
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const S2Shift sh = bshift[i * H + h];
                const S2Rec& rec = brec[i * H + h];
#pragma unroll
                for (int r8 = 0; r8 < S2_H; ++r8)
                    if (h * S2_H + r8 == sub) { w = sh.w[r8]; imp = rec.imp[r8]; }
            }
        };

        // Window of row i for this wave: the largest and smallest shift of the
        // candidates it offers to the task (no candidate: any window will do).
        auto window_of = [&](int i, int& maxs, int& mins) __attribute__((always_inline)) {
            if (full) {
                const S2Info inf = binfo[i];
                maxs = max(inf.maxs, 0);
                mins = inf.maxs < 0 ? 0 : inf.mins;
            } else {
                int w;
                float imp;
                one_row_of(i, w, imp);
                maxs = mins = max(w, 0);
            }
        };

        // Start the copy of the window of row i into ring slot `slot` of KU units
        // of 128 floats: exactly (KU + 1) / 2 copy instructions, whatever the row
        // (whole copies of 256 floats by all lanes, and for an odd KU one of 128
        // floats by the lower half of the wave).
        auto issue_row = [&](auto ku_c, int i, int slot, int maxs, int mins) __attribute__((always_inline)) {
            constexpr int KU = decltype(ku_c)::value;
            constexpr int SLOTF = KU * S2W_UNIT;
            constexpr int NFULL = KU / 2;
            constexpr bool HALF = (KU & 1) != 0;
            // (the lane number is taken afresh here: its multiples are two instructions
            //  to recompute and would otherwise occupy registers throughout the task)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int lo = tW - maxs;
            const int lo4 = lo & ~3;                               // floor to a multiple of 4
            const int n4 = (WV + maxs - mins + (lo - lo4) + 3) & ~3;   // cells needed, in floats (<= SLOTF)
            const int last = min(tmaxg, lo4 + n4 - 4);             // last cell worth fetching
            const float* row = Mb + (size_t)i * P;
            float* dst = ring + slot * SLOTF;
            if (lo4 >= 0) {
                // (wave-uniform base plus an unsigned 32-bit byte offset per lane;
                //  lo4 <= last because the wave has a column below P)
                const char* base = (const char*)(row + lo4);
                const unsigned lastoff = (unsigned)(last - lo4) * 4u;
#pragma unroll
                for (int k = 0; k < NFULL; ++k) {
                    const unsigned off = min((unsigned)(1024 * k + 16 * ln), lastoff);
                    __builtin_amdgcn_global_load_lds((const float*)(base + off),
                                                     (lds_void*)(dst + 256 * k), 16, 0,
                                                     DMA_AGENT_SCOPE);
                }
                if constexpr (HALF) {
                    const unsigned off = min((unsigned)(1024 * NFULL + 16 * ln), lastoff);
                    lds_load16_if(ln < 32, (const float*)(base + off), dst + 256 * NFULL);
                }
            } else {
#pragma unroll
                for (int k = 0; k < NFULL; ++k) {
                    const int tp = min(lo4 + 256 * k + 4 * ln, last);
                    const float* src = tp < 0 ? ninf : row + tp;
                    __builtin_amdgcn_global_load_lds(src, (lds_void*)(dst + 256 * k), 16, 0,
                                                     DMA_AGENT_SCOPE);
                }
                if constexpr (HALF) {
                    const int tp = min(lo4 + 256 * NFULL + 4 * ln, last);
                    lds_load16_if(ln < 32, tp < 0 ? ninf : row + tp, dst + 256 * NFULL);
                }
            }
        };

        // Relax the eight rows h*8 .. h*8+7 of the group from the row whose
        // window sits at `base` (byte address of this lane's column u = 0 at
        // offset 0) with the operands of `rec`.  A candidate whose shift
        // exceeds every column of the task reads the part of the window below
        // column 0 (-inf); a missing candidate adds -inf to whatever its cell
        // holds: neither needs a test here.  LDS reads run one row ahead of
        // the arithmetic.
        auto relax_half = [&](auto hh, const char* base, const S2Rec& rec, uint32_t vi)
                              __attribute__((always_inline)) {
            constexpr int h = decltype(hh)::value;
            float mcur[U], mnxt[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                mcur[u] = *(const float*)(base + rec_off4(rec, 0) + 256 * u);
#pragma unroll
            for (int r8 = 0; r8 < S2_H; ++r8) {
                constexpr int unused = 0;
                (void)unused;
                if (r8 + 1 < S2_H) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        mnxt[u] = *(const float*)(base + rec_off4(rec, r8 + 1) + 256 * u);
                }
                const float imp = rec.imp[r8];
                float cand[U];
#pragma unroll
                for (int u = 0; u < U; ++u) cand[u] = mcur[u] + imp;
                relax_cell<0, STORE_K>(best[h * S2_H + r8][0], argp[h * S2_H + r8], cand[0], vi);
                relax_cell<1, STORE_K>(best[h * S2_H + r8][1], argp[h * S2_H + r8], cand[1], vi);
                relax_cell<2, STORE_K>(best[h * S2_H + r8][2], argp[h * S2_H + r8], cand[2], vi);
                relax_cell<3, STORE_K>(best[h * S2_H + r8][3], argp[h * S2_H + r8], cand[3], vi);
#pragma unroll
                for (int u = 0; u < U; ++u) mcur[u] = mnxt[u];
            }
        };
        // Two predecessors at once (rows a and a + 1, windows at byte offsets baseA and
        // baseB from this lane's place in the ring, lbase): each cell is offered both
        // candidates in one update (PairCell), and the byte that is recorded is the
        // number of the pair (a / 2).  Which of the two it was is settled once per
        // cell after the last predecessor (resolve_pairs).  The operands of the
        // group's rows are taken from the two rows' records a quarter (four rows: 6
        // scalar registers per record) at a time, the next quarter while the current
        // one is in use, so that few scalar registers are live; qa and qb arrive with
        // the first quarter this step needs and leave with the first quarter that the
        // next step needs of the rows whose records start at nextA and nextB.  LDS
        // reads run one row ahead of the arithmetic.
        struct Quarter { uint32_t offp[2]; float imp[4]; };
        auto load_quarter = [&](const S2Rec* row, auto kk) __attribute__((always_inline)) {
            constexpr int k = decltype(kk)::value;         // quarter of the row's R / 4
            const S2Rec& r = row[k / 2];
            Quarter q;
            q.offp[0] = r.offp[2 * (k & 1)];
            q.offp[1] = r.offp[2 * (k & 1) + 1];
#pragma unroll
            for (int x = 0; x < 4; ++x) q.imp[x] = r.imp[4 * (k & 1) + x];
            return q;
        };
        auto quarter_off4 = [](const Quarter& q, int x) __attribute__((always_inline)) {
            return (x & 1) ? (int)(q.offp[x >> 1] >> 16) : (int)(q.offp[x >> 1] & 0xFFFFu);
        };
        // step_c: the kind of the step (see PairCell): which way it goes through the
        // rows, and hence which quarter comes first.
        auto relax_pair_rows = [&](auto step_c, int baseA, int baseB, const S2Rec* rowA,
                                   const S2Rec* rowB, Quarter& qa, Quarter& qb, const S2Rec* nextA,
                                   const S2Rec* nextB, uint32_t vc) __attribute__((always_inline)) {
            static_assert(U == 4, "two halves of two columns per row");
            constexpr int STEP = decltype(step_c)::value;
            constexpr int NQU = R / 4;
            constexpr int K0 = STEP == 0 ? 0 : NQU - 1;     // first quarter of this step
            constexpr int R0 = STEP == 0 ? 0 : R - 1;       // and its first row
            Quarter QA[NQU + 1], QB[NQU + 1];               // [NQU]: for the step that follows
            QA[K0] = qa;
            QB[K0] = qb;
            // (reads a whole row ahead, two columns of each window per instruction:
            //  three buffers of half a row)
            float av[3][2], bv[3][2];
            const char* rowa = lbase + (baseA + quarter_off4(QA[K0], R0 & 3));
            const char* rowb = lbase + (baseB + quarter_off4(QB[K0], R0 & 3));
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                av[0][c] = *(const float*)(rowa + 256 * c);
                bv[0][c] = *(const float*)(rowb + 256 * c);
                av[1][c] = *(const float*)(rowa + 256 * (2 + c));
                bv[1][c] = *(const float*)(rowb + 256 * (2 + c));
            }
            static_for<R>([&](auto nn) __attribute__((always_inline)) {
                constexpr int n = decltype(nn)::value;      // n-th row of this step
                constexpr int rr = STEP == 0 ? n : R - 1 - n;
                constexpr int k = rr / 4, x = rr % 4;
                constexpr int b0 = (2 * n) % 3, b1 = (2 * n + 1) % 3, b2 = (2 * n + 2) % 3;
                if constexpr (n % 4 == 0) {
                    // the operands of the four rows after these four
                    if constexpr (n + 4 < R) {
                        constexpr int kn = STEP == 0 ? k + 1 : k - 1;
                        QA[kn] = load_quarter(rowA, std::integral_constant<int, kn>{});
                        QB[kn] = load_quarter(rowB, std::integral_constant<int, kn>{});
                    } else {
                        constexpr int kn = STEP == 0 ? NQU - 1 : 0;   // the other kind comes next
                        QA[NQU] = load_quarter(nextA, std::integral_constant<int, kn>{});
                        QB[NQU] = load_quarter(nextB, std::integral_constant<int, kn>{});
                    }
                }
                const float ia = QA[k].imp[x], ib = QB[k].imp[x];
                // columns 0, 1 of the next row on their way, columns 0, 1 relaxed
                if constexpr (n + 1 < R) {
                    constexpr int r2 = STEP == 0 ? rr + 1 : rr - 1;
                    rowa = lbase + (baseA + quarter_off4(QA[r2 / 4], r2 & 3));
                    rowb = lbase + (baseB + quarter_off4(QB[r2 / 4], r2 & 3));
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        av[b2][c] = *(const float*)(rowa + 256 * c);
                        bv[b2][c] = *(const float*)(rowb + 256 * c);
                    }
                }
                if constexpr (STORE_K) {
                    PairCell<STEP, rr, 0>::run(best[rr][0], argp[rr], av[b0][0] + ia, bv[b0][0] + ib, vc);
                    PairCell<STEP, rr, 1>::run(best[rr][1], argp[rr], av[b0][1] + ia, bv[b0][1] + ib, vc);
                } else {
                    // values only: one three-way maximum per two candidates
                    max_cand2(best[rr][0], av[b0][0] + ia, bv[b0][0] + ib);
                    max_cand2(best[rr][1], av[b0][1] + ia, bv[b0][1] + ib);
                }
                // columns 2, 3 of the next row on their way, columns 2, 3 relaxed
                if constexpr (n + 1 < R) {
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        av[b0][c] = *(const float*)(rowa + 256 * (2 + c));
                        bv[b0][c] = *(const float*)(rowb + 256 * (2 + c));
                    }
                }
                if constexpr (STORE_K) {
                    PairCell<STEP, rr, 2>::run(best[rr][2], argp[rr], av[b1][0] + ia, bv[b1][0] + ib, vc);
                    PairCell<STEP, rr, 3>::run(best[rr][3], argp[rr], av[b1][1] + ia, bv[b1][1] + ib, vc);
                } else {
                    max_cand2(best[rr][2], av[b1][0] + ia, bv[b1][0] + ib);
                    max_cand2(best[rr][3], av[b1][1] + ia, bv[b1][1] + ib);
                }
            });
            qa = QA[NQU];
            qb = QB[NQU];
        };
        // After the last predecessor below the group every arg-max byte holds a
        // pair number c (or DPC_NOARG).  The arg-max is 2c if that row's candidate
        // reproduces the cell bit for bit (the lower index wins a tie), else 2c + 1.
        // A pair whose second row is not below the group holds its first row alone.
        // tab[c * R + rr] = (4 Topt, I)[2c][j0 + rr], filled by the workgroup (no
        // candidate: a latency no budget reaches).  Two rows at a time in two
        // passes, so that the loads of a pass are in flight together.  A cell whose
        // even candidate does not exist gets +inf to compare with, which equals no
        // maximum.
        struct PairOp { int32_t w4; float imp; };
        auto resolve_pairs = [&](const PairOp* tab, int npairs) __attribute__((always_inline)) {
            // (uniform base plus an unsigned 32-bit byte offset per lane: a pair task
            //  has a table of M smaller than 4 GB and fewer than 2^20 budgets)
            const char* Mc = (const char*)Mb;
            const uint32_t p8 = 8u * (uint32_t)P;
            constexpr int RB = 2;
#pragma unroll
            for (int r0 = 0; r0 < R; r0 += RB) {
                if (r0 >= hq) break;                   // (row slots past the group's rows hold nothing)
                float mv[RB][U];
                const PairOp* ent[RB][U];
#pragma unroll
                for (int p = 0; p < RB; ++p) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t c = min((argp[r0 + p] >> (8 * u)) & 0xFFu, (uint32_t)npairs - 1u);
                        ent[p][u] = tab + (c * R + r0 + p);
                        const int w4 = ent[p][u]->w4;
                        const int tc4 = 4 * min(tS + tl0 + 64 * u, P - 1);   // (cells past the table are never stored)
                        const uint32_t off = __umul24(c, p8) + (uint32_t)(tc4 - w4);
                        mv[p][u] = w4 <= tc4 ? ld_agent((const float*)(Mc + off)) : INFINITY;
                    }
                }
#pragma unroll
                for (int p = 0; p < RB; ++p) {
                    uint32_t odd = 0;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const bool first = mv[p][u] + ent[p][u]->imp == best[r0 + p][u];
                        odd |= first ? 0u : 1u << (8 * u);
                    }
                    // (pair numbers are below 128: a byte with its top bit set is DPC_NOARG and stays)
                    const uint32_t none = ((argp[r0 + p] & 0x80808080u) >> 7) * 0xFFu;
                    argp[r0 + p] = ((argp[r0 + p] << 1) & 0xFEFEFEFEu) | odd | none;
                }
            }
        };
        // The same for a one-row task: only row `sub` of the group, at one shift.
        auto relax_one = [&](int i, int slot, int slotf) __attribute__((always_inline)) {
            int w;
            float imp;
            one_row_of(i, w, imp);
            if (w < 0) return;
            const int delta = (tS - w) & 3;
            const float* base = (const float*)(lbase + (slot * slotf + delta) * 4);
            float cand[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cand[u] = base[64 * u] + imp;
            const uint32_t vi = (uint32_t)i;
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                if (rr != sub) continue;
                relax_cell<0, STORE_K>(best[rr][0], argp[rr], cand[0], vi);
                relax_cell<1, STORE_K>(best[rr][1], argp[rr], cand[1], vi);
                relax_cell<2, STORE_K>(best[rr][2], argp[rr], cand[2], vi);
                relax_cell<3, STORE_K>(best[rr][3], argp[rr], cand[3], vi);
            }
        };

        // The rows prev_row0 .. ilimit-1 are written by the tasks of entry `prev`,
        // which may still be running: a wave waits for them right before it
        // starts the copy of row prev_row0, by which time most of its work on
        // the rows below is done.  A wait that runs out sets the error word and
        // goes on (every access stays in bounds whatever the rows hold).
        auto wait_prev = [&]() __attribute__((always_inline)) {
            const uint32_t* flag = &done[prev];
            const long long start = wall_clock64();
            for (uint32_t spin = 0; ld_uniform(flag) < prev_cnt; ++spin) {
                if ((spin & 15u) == 15u) {
                    if (ld_uniform(&hdr->error) != 0) break;
                    if (wall_clock64() - start > wait_limit) {
                        if (lane == 0)
                            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
                __builtin_amdgcn_s_sleep(2);
            }
        };

        // whole group, smallest windows, table of M below 4 GB: two predecessors per step
        const bool pair_task = PAIRS && full && s2_ring_slots(RINGF, spread) == 5 &&
                               (long long)ld * P < (1LL << 30) && P < (1 << 20);
        // ---------------- off-diagonal part: rows i < ilimit ----------------
        // The part itself, compiled once per ring geometry: NSL slots of KU units,
        // NLD copy instructions per row, D = NSL - 1 rows ahead.
        auto offdiag = [&](auto nld_c, auto nsl_c) __attribute__((always_inline)) {
            constexpr int KU = decltype(nld_c)::value;
            constexpr int NSL = decltype(nsl_c)::value;
            constexpr int NLD = (KU + 1) / 2;
            constexpr int SLOTF = KU * S2W_UNIT;
            constexpr int D = NSL - 1;
            static_assert(NSL * SLOTF <= RINGF, "the slots fit the ring");
            static_assert(D >= 1 && D * NLD <= 10, "the counted wait covers at most 10 loads");
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < ilimit) {
                    if (d == prev_row0) wait_prev();
                    int maxs, mins;
                    window_of(d, maxs, mins);
                    issue_row(nld_c, d, d, maxs, mins);
                }
            int slot = 0;                              // ring slot of row i
            int ahead = D;                             // ring slot of row i + D
            if constexpr (PAIRS && NSL == 5) {
              if (pair_task) {
                // Two predecessor rows per step.  Row r sits in ring slot r mod 5;
                // while rows a and a + 1 are relaxed the copies of a + 2, a + 3 and
                // a + 4 are in flight.  The window of row r + 4 is in the record of
                // row r (the pack kernel looks 4 rows ahead for these groups).
                const S2Rec* rowA = brec;              // records of rows a and a + 1
                const S2Rec* rowB = brec + min(1, L) * H;
                Quarter qa = load_quarter(rowA, std::integral_constant<int, 0>{});
                Quarter qb = load_quarter(rowB, std::integral_constant<int, 0>{});
                // (largest shift, then the window of the row four rows on)
                uint32_t pa0 = rowA->pad[0], pa1 = rowA->pad[1], pa2 = rowA->pad[2];
                uint32_t pb0 = rowB->pad[0], pb1 = rowB->pad[1], pb2 = rowB->pad[2];
                int sa = 0;                            // ring slot of row a
                int pw_max = 0, pw_min = 0;            // window of row a + 3
                int a = 0;
                auto pair_step = [&](auto step_c) __attribute__((always_inline)) {
                    const int s3 = sa + 3 >= NSL ? sa + 3 - NSL : sa + 3;
                    const int s4 = sa + 4 >= NSL ? sa + 4 - NSL : sa + 4;
                    if (a >= 2 && a + 3 < ilimit) {
                        if (a + 3 == prev_row0) wait_prev();
                        issue_row(nld_c, a + 3, s3, pw_max, pw_min);
                    }
                    if (a + 4 < ilimit) {
                        if (a + 4 == prev_row0) wait_prev();
                        issue_row(nld_c, a + 4, s4, (int)pa1, (int)pa2);
                    }
                    // rows up to min(ilimit, a + 5) - 1 have been issued; a and a + 1 must have landed
                    wait_vm((min(ilimit, a + 5) - (a + 2)) * NLD);
                    asm volatile("" ::: "memory");
                    pw_max = (int)pb1;
                    pw_min = (int)pb2;
                    const int sb = sa + 1 >= NSL ? 0 : sa + 1;
                    const int dA = (tS - (int)pa0) & 3;
                    const int dB = (tS - (int)pb0) & 3;
                    const int baseA = (sa * SLOTF + dA) * 4;
                    const int baseB = (sb * SLOTF + dB) * 4;
                    // Workgroups of 8 or 16 waves have two or four waves on every SIMD,
                    // which all reach the barrier in front of the diagonal part before any
                    // goes on: the issue priority goes round them from step to step, so
                    // that they advance together instead of finishing one after the other
                    // (the last ones alone on their SIMD).
                    if constexpr (NW >= 8) rotate_priority(((uint32_t)a >> 1) + (uint32_t)(wave >> 2));
                    const uint32_t vc = (uint32_t)a >> 1;
                    const S2Rec* nextA = brec + min(a + 2, L) * H;
                    const S2Rec* nextB = brec + min(a + 3, L) * H;
                    const uint32_t na0 = nextA->pad[0], na1 = nextA->pad[1], na2 = nextA->pad[2];
                    const uint32_t nb0 = nextB->pad[0], nb1 = nextB->pad[1], nb2 = nextB->pad[2];
                    relax_pair_rows(step_c, baseA, baseB, rowA, rowB, qa, qb, nextA, nextB, vc);
                    rowA = nextA;
                    rowB = nextB;
                    pa0 = na0; pa1 = na1; pa2 = na2;
                    pb0 = nb0; pb1 = nb1; pb2 = nb2;
                    sa = sa + 2 >= NSL ? sa + 2 - NSL : sa + 2;
                    a += 2;
                };
                // (two steps per trip, one of each kind: see PairCell)
                while (a + 3 < ilimit) {
                    pair_step(std::integral_constant<int, 0>{});
                    pair_step(std::integral_constant<int, 1>{});
                }
                if (a + 1 < ilimit) pair_step(std::integral_constant<int, 0>{});
                if (a < ilimit) {
                    // an odd number of rows: the last one is a pair of its own
                    wait_vm(0);
                    asm volatile("" ::: "memory");
                    const int dA = (tS - (int)pa0) & 3;
                    const char* base = lbase + (sa * SLOTF + dA) * 4;
                    const uint32_t vc = (uint32_t)a >> 1;
                    const S2Rec last0 = rowA[0];
                    relax_half(std::integral_constant<int, 0>{}, base, last0, vc);
                    if constexpr (H == 2) {
                        const S2Rec last1 = rowA[H - 1];
                        relax_half(std::integral_constant<int, 1>{}, base, last1, vc);
                    }
                }
                return;
              }
            }
            if (full) {
                S2Rec cur[H];
#pragma unroll
                for (int h = 0; h < H; ++h) cur[h] = brec[h];
                for (int i = 0; i < ilimit; ++i) {
                    const int inext = min(i + 1, L) * H;
                    // the loads of the D rows ahead stay in flight; past the last
                    // row there is nothing left to start and nothing to leave
                    if (i + D < ilimit) {
                        if (i + D == prev_row0) wait_prev();
                        issue_row(nld_c, i + D, ahead, (int)cur[0].pad[1], (int)cur[0].pad[2]);
                        wait_vm(D * NLD);
                    } else {
                        wait_vm(0);
                    }
                    asm volatile("" ::: "memory");             // row i has landed
                    const int delta = (tS - (int)cur[0].pad[0]) & 3;   // alignment slack of the window
                    const char* base = lbase + (slot * SLOTF + delta) * 4;
                    const uint32_t vi = cur[0].pad[3];
                    if constexpr (H == 1) {
                        const S2Rec nxt = brec[inext];
                        relax_half(std::integral_constant<int, 0>{}, base, cur[0], vi);
                        cur[0] = nxt;
                    } else {
                        // the operands of each half are fetched for the next row as
                        // soon as the half has been used
                        relax_half(std::integral_constant<int, 0>{}, base, cur[0], vi);
                        const S2Rec nxt0 = brec[inext];
                        relax_half(std::integral_constant<int, 1>{}, base, cur[H - 1], vi);
                        cur[H - 1] = brec[inext + H - 1];
                        cur[0] = nxt0;
                    }
                    ahead = slot;
                    slot = slot + 1 == NSL ? 0 : slot + 1;
                }
            } else if constexpr (NSL == 5) {
                // (a one-row task has one shift per predecessor: the smallest window)
                for (int i = 0; i < ilimit; ++i) {
                    if (i + D < ilimit) {
                        if (i + D == prev_row0) wait_prev();
                        int maxs, mins;
                        window_of(i + D, maxs, mins);
                        issue_row(nld_c, i + D, ahead, maxs, mins);
                        wait_vm(D * NLD);
                    } else {
                        wait_vm(0);
                    }
                    asm volatile("" ::: "memory");
                    relax_one(i, slot, SLOTF);
                    ahead = slot;
                    slot = slot + 1 == NSL ? 0 : slot + 1;
                }
            }
        };
        if (!wave_idle) {
            // as many slots as hold the windows of the task: 5, 3 or 2, each as large as the ring allows
            constexpr int U5 = s2_slot_units_max(RINGF, 5), U3 = s2_slot_units_max(RINGF, 3),
                          U2 = s2_slot_units_max(RINGF, 2);
            const int need = s2_units_needed(full ? spread : 0);
            using std::integral_constant;
            if (need <= U5) offdiag(integral_constant<int, U5>{}, integral_constant<int, 5>{});
            else if (need <= U3) offdiag(integral_constant<int, U3>{}, integral_constant<int, 3>{});
            else offdiag(integral_constant<int, U2>{}, integral_constant<int, 2>{});
        }
        if constexpr (NW >= 8) rotate_priority(0u);
        if (!full) {
            // ---------------- a one-row task only has its row to store ----------------
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                if (rr != sub) continue;
                store_row(j0 + rr, rr);
            }
        } else {
            // operands of the even rows below the group for the pair settlement: the
            // first ones are fetched before the barrier (whose wait covers their
            // latency); all go behind the two diagonal slots after it
            constexpr int TRIPS = (PAIR_TAB + NT - 1) / NT;
            constexpr int EARLY = TRIPS < 2 ? TRIPS : 2;
            const int nent = ((j0 + 1) >> 1) * R;              // pairs (2c, 2c + 1) with 2c < j0
            auto pair_operands = [&](int k) __attribute__((always_inline)) {
                const int en = min(tid + k * NT, nent - 1);
                const int c = en / R, rr = en - c * R;
                int32_t w;
                PairOp o;
                Topt.operands(I, b, ld, 2 * c, min(j0 + rr, L), w, o.imp);
                o.w4 = w >= 0 && w < P ? 4 * w : 0x7FFFFFFF;       // (the pack kernel's rule)
                return o;
            };
            PairOp early[EARLY];
            if constexpr (PAIRS && STORE_K) {
                if (pair_task) {
#pragma unroll
                    for (int k = 0; k < EARLY; ++k)
                        if (k * NT < nent) early[k] = pair_operands(k);
                }
            }
            __syncthreads();                           // every ring is idle: the slots below lie over them
            if constexpr (PAIRS && STORE_K) {
                if (pair_task) {
                    PairOp* tab = (PairOp*)(lds + 2 * DSLOTW);
                    PairOp late[TRIPS - EARLY + 1];
#pragma unroll
                    for (int k = EARLY; k < TRIPS; ++k)
                        if (k * NT < nent) late[k - EARLY] = pair_operands(k);
#pragma unroll
                    for (int k = 0; k < EARLY; ++k)
                        if (tid + k * NT < nent) tab[tid + k * NT] = early[k];
#pragma unroll
                    for (int k = EARLY; k < TRIPS; ++k)
                        if (tid + k * NT < nent) tab[tid + k * NT] = late[k - EARLY];
                    __syncthreads();
                    if (!wave_idle) resolve_pairs(tab, (j0 + 1) >> 1);
                }
            }
            if (tS == 0) {
                // first strip: what lies to the left of column 0 does not exist
                for (int x = tid; x < 2 * DMAX; x += NT) {
                    const int sl = x / DMAX;
                    lds[sl * DSLOTW + (x - sl * DMAX)] = NINF;
                }
            }
            // ---------------- diagonal part and output ----------------
            // Straight-line code for every wave and every row of the group: a row
            // past the last layer has no candidates in the records (importance
            // -inf) and is not stored, and a wave past the last column relaxes
            // cells that are never stored.
            S2Rec drec[H];                             // operands of the group's own row rr
#pragma unroll
            for (int h = 0; h < H; ++h) drec[h] = brec[min(j0, L) * H + h];
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const int j = j0 + rr;
                if (rr < hq) store_row(j, rr);
                if (rr + 1 < R) {
                    // row j feeds the rows below it through an LDS slot: own column t
                    // at slot position DMAX + (t - tS).  Two slots alternate: a slot
                    // is written again only after the barrier that follows the reads
                    // of its previous contents.
                    float* slot = lds + (rr & 1) * DSLOTW;
#pragma unroll
                    for (int u = 0; u < U; ++u) slot[DMAX + tl0 + 64 * u] = best[rr][u];
                    __syncthreads();
                    const int maxs = (int)drec[0].pad[0];
                    const uint32_t vj = (uint32_t)j;
#pragma unroll
                    for (int r2 = rr + 1; r2 < R; ++r2) {
                        // shifts inside a group are at most DMAX: a shift beyond
                        // the task's last column can only occur in the first
                        // strip, whose pad holds -inf
                        const S2Rec& rec = drec[r2 / S2_H];
                        const int w = maxs - (rec_off4(rec, r2 % S2_H) >> 2);
                        const float imp = rec.imp[r2 % S2_H];
                        const float* sp = &slot[DMAX - w + tl0];
                        float cand[U];
#pragma unroll
                        for (int u = 0; u < U; ++u) cand[u] = sp[64 * u] + imp;
                        relax_cell<0, STORE_K>(best[r2][0], argp[r2], cand[0], vj);
                        relax_cell<1, STORE_K>(best[r2][1], argp[r2], cand[1], vj);
                        relax_cell<2, STORE_K>(best[r2][2], argp[r2], cand[2], vj);
                        relax_cell<3, STORE_K>(best[r2][3], argp[r2], cand[3], vj);
                    }
                    // operands of the next row of the group
#pragma unroll
                    for (int h = 0; h < H; ++h) drec[h] = brec[min(j + 1, L) * H + h];
                }
            }
        }
        // ---- the task is complete once every wave's stores are acknowledged;
        //      wave 0 publishes it at the top of the loop
        wait_vm(0);
        __syncthreads();                               // (also: the LDS is free again)
        publish = e;
    }
}

// gated / want / decide: see launch_stage2_prepare; the main kernel is gated on
// `want` when either is set
template <int R, int NW, int RINGF, int DMAX, int WPE>
static hipError_t launch_wave_cfg(int B, int L, int P, ToptRef Topt, const float* I, float* M,
                                  uint8_t* K, void* workspace, int num_cu, hipStream_t st,
                                  bool gated = false, uint32_t want = 0, bool decide = false)
{
    constexpr int WCAP = NW * 256;
    const int NQ = (L + R - 1) / R;
    const S2Layout lay = s2_layout(B, L, P, R);
    char* base = (char*)workspace;
    S2Header* hdr = (S2Header*)base;
    uint32_t* done = (uint32_t*)(base + lay.done_off);
    S2Entry* entries = (S2Entry*)(base + lay.entry_off);
    S2Task* tasks = (S2Task*)(base + lay.task_off);
    S2Rec* recs = (S2Rec*)(base + lay.rec_off);
    S2Info* infos = (S2Info*)(base + lay.info_off);
    S2Shift* shifts = (S2Shift*)(base + lay.shift_off);

    // ghost columns cost recomputation: at most half of a task (beyond that the
    // group runs row by row), and the chain of shifts must fit the pad in front
    // of a diagonal slot
    const int gmax = std::min(DMAX, WCAP / 2);
    hipError_t e = launch_stage2_prepare(B, L, P, R, Topt, I, M, K, workspace, gmax, s2_max_spread(RINGF),
                                         DMAX, WCAP, -4, RINGF, st, gated, want, decide);
    if (e != hipSuccess) return e;
    const S2Gate gate{gated || decide ? &hdr->choice : nullptr, want};

    // resident workgroups per compute unit: WPE waves per SIMD, 4 SIMDs
    constexpr int wg_per_cu = (WPE * 4) / NW;
    static_assert(wg_per_cu >= 1, "a workgroup must fit one compute unit");
    int grid = num_cu * wg_per_cu;
    // A table that fits one task per row group is B independent chains of
    // tasks.  Two workgroups per chain are what can work at once (one finishes a
    // group while the next has started on the rows below it); more only wait.
    // Any number is safe: a ticket only ever waits for lower tickets.
    if (P <= WCAP) {
        const long long n = B;
        const long long fit = 2 * n;
        if (fit < grid) grid = (int)fit;
    }
    const long long wait_limit = 500000000LL;      // 5 s of the 100 MHz wall clock
    if (K)
        hipLaunchKernelGGL((stage2_wave_kernel<R, NW, RINGF, DMAX, WPE, true>), dim3(grid),
                           dim3(NW * 64), 0, st, B, L, P, M, K, hdr, done, entries, tasks, recs,
                           infos, shifts, NQ, wait_limit, gate, Topt, I);
    else
        hipLaunchKernelGGL((stage2_wave_kernel<R, NW, RINGF, DMAX, WPE, false>), dim3(grid),
                           dim3(NW * 64), 0, st, B, L, P, M, K, hdr, done, entries, tasks, recs,
                           infos, shifts, NQ, wait_limit, gate, Topt, I);
    return hipGetLastError();
}

// groups of 8 rows (shapes 1-4) or 16 rows (5, 6, 8): waves per task, floats of a
// wave's ring, largest shift inside a group, waves per SIMD
static hipError_t launch_wave_shape(int shape, int B, int L, int P, ToptRef Topt, const float* I,
                                    float* M, uint8_t* K, void* workspace, int num_cu, hipStream_t st,
                                    bool gated, uint32_t want, bool decide)
{
    switch (shape) {
        case 1: return launch_wave_cfg<8, 4, 1920, 764, 5>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 2: return launch_wave_cfg<8, 8, 1920, 764, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 3: return launch_wave_cfg<8, 2, 1920, 764, 5>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 4: return launch_wave_cfg<8, 1, 1920, 764, 5>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 5: return launch_wave_cfg<16, 4, 2560, 764, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 6: return launch_wave_cfg<16, 8, 2560, 764, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        case 8: return launch_wave_cfg<16, 16, 2560, 764, 4>(B, L, P, Topt, I, M, K, workspace, num_cu, st, gated, want, decide);
        default: return hipErrorInvalidValue;
    }
}

bool stage2_wave_shape_known(int shape) { return (shape >= 1 && shape <= 6) || shape == 8; }

// shape 0: chosen from the problem size (below); otherwise one of the task
// shapes of launch_wave_shape, whatever the size (tests and measurements)
hipError_t launch_stage2_wave(int B, int L, int P, ToptRef Topt, const float* I, float* M,
                              uint8_t* K, void* workspace, int num_cu, int shape, hipStream_t st)
{
    // a window cell may read up to three floats past the end of a row
    if (P < 16) return hipErrorInvalidValue;
    if (shape != 0)
        return launch_wave_shape(shape, B, L, P, Topt, I, M, K, workspace, num_cu, st, false, 0u, false);
    // Task shape.  Groups of 8 rows: the narrowest task that covers a narrow
    // table, 2048 columns per task for wide ones.  Chains of 64 layers and more
    // run in groups of 16 rows where the table is wider than 512 budgets: they
    // halve the number of times every row of M is read back.  Their tasks are as
    // wide as the table where 4, 8 or 16 waves cover it (no strip edges at all
    // then), and 16 waves wide beyond that (4096 columns: a quarter of the ghost
    // columns of 1024-column strips), except where the tasks of a level would
    // fill the chip's compute units a whole number of times and a little more:
    // then the finer 4-wave tasks.  The whole-width shapes of 8 and 16 waves also
    // win for shorter chains when the batch fills the chip with such tasks.
    // Measured on chains of 32 to 200 layers at 1000 to 16000 budgets, batches
    // of 32 to 1024, and on the 109-layer chains of the extended solver.
    const int narrow = P <= 256 ? 4 : P <= 512 ? 3 : P <= 1536 ? 1 : 2;
    int wide = 0;
    if (P > 512 && L >= 64) {
        if (P <= 1024) wide = 5;
        else if (P <= 2048) wide = 6;
        else if (P <= 4096) wide = 8;
        else {
            // (the ghost width is only known on the device: 128 columns assumed)
            const long long strips = 1 + ((long long)P - 4096 + 3967) / 3968;
            const long long tasks = strips * B;
            const long long rounds = (tasks + num_cu - 1) / num_cu, rem = tasks % num_cu;
            wide = (rounds >= 2 && rem != 0 && 4 * rem < num_cu) ? 5 : 8;
        }
    } else if (P > 512 && L > 16) {
        if (P > 1536 && P <= 2048 && B >= 2LL * num_cu) wide = 6;
        else if (P > 2048 && P <= 4096 && B >= num_cu) wide = 8;
    }
    if (wide == 0)
        return launch_wave_shape(narrow, B, L, P, Topt, I, M, K, workspace, num_cu, st, false, 0u, false);
    // Groups of 16 rows need the shifts of 16 consecutive layers to fit a window
    // and a ghost region; whether they do is only known on the device.  Prepare
    // them, let the device decide, and queue the 8-row shape behind it: of the
    // two main kernels one returns at once.
    hipError_t e = launch_wave_shape(wide, B, L, P, Topt, I, M, K, workspace, num_cu, st, false, 0u, true);
    if (e != hipSuccess) return e;
    return launch_wave_shape(narrow, B, L, P, Topt, I, M, K, workspace, num_cu, st, true, 1u, false);
}

}  // namespace dpc
