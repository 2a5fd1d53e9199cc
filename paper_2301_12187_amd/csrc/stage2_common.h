// Declarations shared by the persistent stage-2 kernels (Algorithm 2 /
// recurrence Eq. 7 of the paper): the workspace layout, the repacked operand
// records and the task table, and the small kernels that build them.
#pragma once
#include <algorithm>
#include <cstddef>
#include <type_traits>
#include "dpc_internal.h"

namespace dpc {

typedef __attribute__((address_space(3))) void lds_void;

constexpr int S2_H = 8;            // rows per operand record; a group has 8 or 16 rows

struct S2Header {
    uint32_t ticket;               // next ticket.  Alone in its 128 bytes: the atomics on it share
    uint32_t pad0[31];             // a cache line with nothing that waiting waves poll
    float ninf[4];                 // byte 128: sixteen bytes of -inf, the source of window
                                   // cells that lie below column 0 (layout kernel)
    uint32_t choice;               // which of two prepared shapes runs (set by the layout
                                   // kernel of the first one)
    uint32_t error;                // set when a bounded wait ran out (dpc_stage2_check)
    uint32_t total;                // number of tasks, written by the layout kernel
    uint32_t pad1[25];
};
static_assert(sizeof(S2Header) == 256, "header is one 256-byte block");
static_assert(offsetof(S2Header, error) == S2_ERROR_WORD_OFFSET, "dpc_stage2_check reads this word");

// A launch can be made conditional on the header's `choice` word: its kernels
// return at once unless the word equals `want` (word == nullptr: unconditional).
struct S2Gate {
    const uint32_t* word;
    uint32_t want;
};
__device__ __forceinline__ bool s2_gate_closed(S2Gate g)
{
    return g.word != nullptr && __hip_atomic_load(g.word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != g.want;
}

struct __attribute__((aligned(64))) S2Rec {
    uint32_t offp[S2_H / 2];       // 4 * (maxs - Topt[i][j0+rr]) as 16-bit halves (rr even: low),
                                   // the byte offset of the candidate in the LDS window of row
                                   // i; 0 where there is no candidate
    float imp[S2_H];               // I[i][j0+rr]; -inf where there is no candidate
    uint32_t pad[S2_H / 2];        // [0]: largest shift of the record; [1], [2]: largest and
                                   // smallest shift of the record `ahead` rows further on
                                   // (0 where a record holds no candidate); [3]: i.  In a
                                   // group of 16 rows the offsets of both records count from
                                   // the largest shift of the sixteen, and so do these
};

// byte offset of candidate rr inside the window of its row
__device__ __forceinline__ int rec_off4(const S2Rec& r, int rr)
{
    return (rr & 1) ? (int)(r.offp[rr >> 1] >> 16) : (int)(r.offp[rr >> 1] & 0xFFFFu);
}

struct S2Shift {
    int32_t w[S2_H];               // Topt[i][j0+rr] itself, -1 where there is no candidate
};                                 // (read by the row-by-row path only)

struct S2Info {
    int32_t mins, maxs;            // over the valid shifts of the record; maxs = -1: none
};

// one entry per (level, instance); level = group * R + row-in-group
struct S2Entry {
    int32_t cnt;                   // number of strips (tasks)
    int32_t prev;                  // entry whose rows this one reads last, -1: none
    int32_t prev_cnt;              // number of tasks of that entry
    int32_t g;                     // >= 0: whole group, ghost width; -1: one row
    int32_t prev_row0;             // first row that entry `prev` writes
    int32_t prev2;                 // the entry before `prev` (all rows below prev_row0 are
    int32_t prev2_cnt;             // final once it is complete), -1: none; its task count
    int32_t spread;                // whole group: largest spread of a predecessor's shifts into it
};

struct S2Task {
    int32_t entry, strip;          // in ticket order
};

struct S2Layout {
    size_t done_off, entry_off, group_off, task_off, rec_off, info_off, shift_off, total;
    long long nentries, maxtasks;
};

S2Layout s2_layout(int B, int L, int P, int R);

// Queues the kernels that prepare a stage-2 launch on `st`: clears the header
// and the completion counters, writes row 0 of M (and K), repacks Topt and I
// into records for row groups of R (8 or 16) rows and decides per group whether it
// runs whole (ghost width <= gmax, every spread <= dspread, every shift inside
// the group <= dpad) or row by row, and lays out the task table for strips of
// `wcap` columns.  `ahead`: see S2Rec::pad; a negative value asks for
// min(-ahead, s2_rows_ahead(ringf, spread of the group)).
// gated: every kernel returns at once unless the header's choice word equals
// `want` (the word survives this call's clearing).  decide: the layout kernel
// sets the choice word to 1 if more than 2 % of the groups have to run row by
// row (so that a second, gated preparation with smaller groups takes over),
// else to 0.
hipError_t launch_stage2_prepare(int B, int L, int P, int R, ToptRef Topt, const float* I,
                                 float* M, uint8_t* K, void* workspace, int gmax, int dspread,
                                 int dpad, int wcap, int ahead, int ringf, hipStream_t st,
                                 bool gated = false, uint32_t want = 0, bool decide = false);

// What the pack kernel records about a group that runs whole: ghost width
// (< 4096) and largest spread, in one non-negative word.
__host__ __device__ __forceinline__ int s2_group_code(int ghost, int spread) { return ghost | (spread << 12); }
__host__ __device__ __forceinline__ int s2_group_ghost(int code) { return code & 0xFFF; }
__host__ __device__ __forceinline__ int s2_group_spread(int code) { return code >> 12; }

// The wave-window kernel keeps, per wave, a ring of `ringf` floats in LDS (2560
// for groups of 16 rows, 1920 for groups of 8: a compile-time constant of the
// kernel).  A window of 256 columns plus `spread` (plus 3 of alignment slack)
// is copied in units of 128 floats (a copy instruction moves 256 floats with
// all lanes or 128 with the lower half of the wave).  The ring holds 5, 3 or 2
// slots, chosen per task from the spread the pack kernel found for the group,
// each as large as the ring allows (3 or 4 units with five slots), and the
// kernel copies 4, 2 or 1 rows ahead of the one it relaxes.
constexpr int S2W_UNIT = 128;
__host__ __device__ __forceinline__ int s2_units_needed(int spread) { return (256 + spread + 3 + S2W_UNIT - 1) / S2W_UNIT; }
// largest slot, in units, when the ring is cut into `slots` slots (8 units at most)
__host__ __device__ constexpr int s2_slot_units_max(int ringf, int slots)
{
    return ringf / (S2W_UNIT * slots) < 8 ? ringf / (S2W_UNIT * slots) : 8;
}
__host__ __device__ __forceinline__ int s2_ring_slots(int ringf, int spread)
{
    const int need = s2_units_needed(spread);
    return need <= s2_slot_units_max(ringf, 5) ? 5 : need <= s2_slot_units_max(ringf, 3) ? 3 : 2;
}
__host__ __device__ __forceinline__ int s2_rows_ahead(int ringf, int spread) { return s2_ring_slots(ringf, spread) - 1; }
// the largest spread a whole-group task can take (two slots)
__host__ __device__ constexpr int s2_max_spread(int ringf) { return S2W_UNIT * s2_slot_units_max(ringf, 2) - 259; }

// Row groups.  Rows 1..L are cut into NQ = ceil(L / R) groups of R rows; when R
// does not divide L the FIRST group is the short one (it has next to no
// predecessors), so that the groups with many predecessors carry no rows that
// do not exist.  A task still spans R row slots: the slots past the rows of a
// short group have no candidates and are never stored.
__host__ __device__ __forceinline__ int s2_group_rows(int L, int R, int q)
{
    return q == 0 ? L - ((L + R - 1) / R - 1) * R : R;
}
__host__ __device__ __forceinline__ int s2_group_first_row(int L, int R, int q)
{
    return q == 0 ? 1 : 1 + (L - ((L + R - 1) / R - 1) * R) + (q - 1) * R;
}

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same for wave-uniform code: every lane loads the word, the value of the
// first lane is used, so what depends on it stays wave-uniform (scalar branches).
__device__ __forceinline__ uint32_t ld_uniform(const uint32_t* p)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)ld_relaxed(p));
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
constexpr int DMA_AGENT_SCOPE = 16;        // cache-policy bit sc1 of the global -> LDS load

// Wait until at most `later` of the vector-memory operations this wave has
// issued are still outstanding.  They complete in order, so this waits for
// everything issued before the last `later` ones.  A smaller number only waits
// longer, so the count is clamped to what is spelled out here.
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
        case 8: __builtin_amdgcn_s_waitcnt(0x0F78); break;
        case 9: __builtin_amdgcn_s_waitcnt(0x0F79); break;
        default: __builtin_amdgcn_s_waitcnt(0x0F7A); break;
    }
}

}  // namespace dpc
