// Stage 1 and stage 2 in one launch for small instances (Algorithms 1 and 2 of
// the paper): the latency path for a single network or a handful of them, where
// the batched kernels are bound by launches and by hand-overs between
// workgroups rather than by arithmetic.
//
// One workgroup per instance, one column t of the budget axis per thread (two
// when P > 1024).  Everything the recurrence of Eq. 7 reads sits in LDS:
//   - a table of candidates, indexed [j][i]: the importance I[i][j] and the
//     LDS byte offset that the shift Topt[i][j] turns into (filled by stage 1,
//     which runs first, one wave per source row);
//   - the rows of M themselves, each preceded by one cell of -inf that every
//     candidate with t < Topt[i][j] is pointed at (address clamp instead of a
//     test).  When not every row fits, the first rows stay in LDS, the two
//     newest rows pass through a small ring of slots, and the rows between
//     are read back from the output array in global memory, a batch of rows
//     at a time, started before the work on the resident rows.
// A row costs one barrier.  Candidates are visited in ascending i and replace
// the maximum only when strictly greater: the lowest arg-max is kept.
//
// With a query list (dpc_solve_fused) the workgroup goes on, in the same
// launch, to recover the sets of the queries that name its instance: its waves
// share the list in chunks of 64 queries, a lane per query finds the ones that
// are the workgroup's, and the wave walks them one after the other
// (backtrack_walk.h) through tables that the workgroup itself has just written.
#include "backtrack_walk.h"
#include "stage1_row.h"
#include "stage2_common.h"

namespace dpc {

struct FsCand { int32_t off; float imp; };      // 8 bytes, read as one LDS access

// LDS access by 32-bit LDS address (the candidate table stores such addresses)
#ifndef DPC_HOST_EMU
typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) char lds_char;
__device__ __forceinline__ float lds_ld(int addr) { return *(const lds_float*)(uintptr_t)(uint32_t)addr; }
__device__ __forceinline__ void lds_st(int addr, float v) { *(lds_float*)(uintptr_t)(uint32_t)addr = v; }
__device__ __forceinline__ int lds_address(char* p) { return (int)(uint32_t)(uintptr_t)(lds_char*)p; }
#else
inline float lds_ld(int addr) { return *(const float*)(emu::g_dyn_lds + addr); }
inline void lds_st(int addr, float v) { *(float*)(emu::g_dyn_lds + addr) = v; }
inline int lds_address(char* p) { return (int)(p - emu::g_dyn_lds); }
#endif

constexpr int FS_RING = 3;                      // LDS slots shared by the rows past the resident ones
constexpr int FS_LIST = 64;                     // entries of a wave's set lists (L <= 63)
constexpr int FS_LIST_BYTES = 16 * 2 * FS_LIST * 4;   // LDS of the query phase: 16 waves, two lists each

// the query list of dpc_solve_fused (Q == 0: none)
struct FsQueries {
    int Q;
    const int32_t* q_inst;
    const int32_t* q_T0;
    int32_t* A;
    int32_t* A_len;
    int32_t* S;
    int32_t* S_len;
    float* obj;
    int32_t* lat;
    int32_t* status;
};

// NR: rows of M that stay in LDS for good (rows 0 .. NR-1).  When NR < L+1 the
// rows from NR on share FS_RING more slots, row i in slot NR + (i - NR) % 3: a
// target row j reads rows j-1 and j-2 there (the third slot is the one row j
// itself is written to) and the rows NR .. j-3 from the output array in global
// memory.
template <int U, bool STORE_K, bool QUERIES>
__global__ __launch_bounds__(1024) void fused_small_kernel(
    int B, int L, int P, int NR, const int32_t* __restrict__ T, const float* __restrict__ I,
    int32_t* Topt, uint8_t* split, float* M, uint8_t* K, FsQueries qs)
{
#ifndef DPC_HOST_EMU
    extern __shared__ __attribute__((aligned(16))) char smem[];
#else  // the CPU emulation build of the tests hands the block over
    char* const smem = emu::g_dyn_lds;
#endif
    constexpr int CH = 24 / U;                          // rows read back from global memory per batch
    constexpr int LB = 8 / U;                           // rows read from LDS per batch
    const int ld = L + 1;
    const int RS = P + 1;                               // floats per LDS row: the -inf cell, then P columns
    // LDS: candidate table [ld][ld] (entry [j][i]), then the slots for rows of
    // M; their space first holds a copy of T for stage 1.  Offsets below are
    // in bytes from the start of the LDS block.
    FsCand* const cand_tab = (FsCand*)smem;
    const int rows0 = lds_address(smem) + ld * ld * (int)sizeof(FsCand);   // LDS address of slot 0
    const int nslots = NR < ld ? NR + FS_RING : NR;
    const int NT = blockDim.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = NT >> 6;
    const int b = blockIdx.x;
    const size_t inst = (size_t)b * ld * ld;
    const float* Ib = I + inst;
    float* Mb = M + (size_t)b * ld * P;
    uint8_t* Kb = STORE_K ? K + (size_t)b * ld * P : nullptr;
    constexpr float NINF = -INFINITY;
    auto slot_of = [&](int i) { return i < NR ? i : NR + (i - NR) % FS_RING; };

    // ---------------- stage 1: wave per source row k; L <= 63, lane = target l ----------------
    int32_t* const Tl = (int32_t*)(smem + ld * ld * sizeof(FsCand));
    for (int x = tid; x < ld * ld; x += NT) Tl[x] = T[inst + x];
    __syncthreads();
    for (int k = wave; k <= L; k += nw) {
        int32_t cur[1], arg[1];
        stage1_row<1, 16, true>(L, Tl, k, lane, cur, arg);
        const int l = lane;
        if (l <= L) {
            const bool upper = l > k;
            Topt[inst + (size_t)k * ld + l] = upper ? cur[0] : 0;
            split[inst + (size_t)k * ld + l] = upper ? (uint8_t)arg[0] : (uint8_t)0;
            if (upper) {
                // a shift of P or more (DPC_INF included) reaches no column: any
                // such shift points every column at the -inf cell
                const int w = max(min(cur[0], P), 0);
                FsCand c;
                c.off = rows0 + (slot_of(k) * RS + 1 - w) * 4;
                c.imp = Ib[k * ld + l];
                cand_tab[l * ld + k] = c;
            }
        }
    }
    __syncthreads();                                    // the copy of T gives way to the rows of M

    // ---------------- stage 2 ----------------
    int tc[U], tc4[U];                                  // this thread's columns, clamped to P-1; times 4
    int t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        t[u] = tid + NT * u;
        tc[u] = min(t[u], P - 1);
        tc4[u] = tc[u] * 4;
    }
    // a wave whose columns all lie beyond the table only takes part in the barriers
    const bool active = wave * 64 < P;
    // row 0: objective +0 at every budget
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (t[u] < P) {
            Mb[t[u]] = 0.0f;
            if (STORE_K) Kb[t[u]] = DPC_NOARG;
            lds_st(rows0 + 4 + t[u] * 4, 0.0f);
        }
    for (int r = tid; r < nslots; r += NT) lds_st(rows0 + r * RS * 4, NINF);
    __syncthreads();

    for (int j = 1; j <= L; ++j) {
        float best[U];
        int arg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { best[u] = NINF; arg[u] = DPC_NOARG; }
        const FsCand* cj = cand_tab + j * ld;
        // candidates i < na and i >= nc come from LDS, the ones between from global memory
        const int na = min(j, NR);
        const int nc = max(na, j - (FS_RING - 1));
        if (active) {
            float pre[CH][U];
            float preimp[CH];
            // start the loads of up to CH rows i0, i0+1, ... < nc from global memory
            auto fetch = [&](int i0) __attribute__((always_inline)) {
                int slot = slot_of(i0);                 // rows from NR on cycle through the ring
#pragma unroll
                for (int a = 0; a < CH; ++a) {
                    // (loads are skipped four rows at a time: a row past the
                    //  last one of a started group reads the last one again)
                    if (i0 + (a & ~3) >= nc) break;
                    const bool past = i0 + a >= nc;
                    const int i = past ? nc - 1 : i0 + a;
                    const FsCand c = cj[i];
                    preimp[a] = c.imp;
                    // the shift, back from the LDS address in the entry
                    const int w = slot * RS + 1 - ((c.off - rows0) >> 2);
                    const float* row = Mb + (size_t)i * P;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int tt = tc[u] - w;
                        const float m = ld_agent(row + max(tt, 0));
                        pre[a][u] = tt >= 0 ? m : NINF;
                    }
                    if (i0 + a + 1 < nc) slot = slot + 1 == NR + FS_RING ? NR : slot + 1;
                }
            };
            auto use = [&](int i0) __attribute__((always_inline)) {
#pragma unroll
                for (int a = 0; a < CH; ++a) {
                    if (i0 + a >= nc) break;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const float v = pre[a][u] + preimp[a];
                        if (v > best[u]) { best[u] = v; arg[u] = i0 + a; }
                    }
                }
            };
            // one candidate from a row in LDS
            auto relax_lds = [&](int i, int slot) __attribute__((always_inline)) {
                const FsCand c = cj[i];                 // the same address in every lane: a broadcast
                const int lo = rows0 + slot * RS * 4;   // the -inf cell of the row's slot
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float v = lds_ld(max(tc4[u] + c.off, lo)) + c.imp;
                    if (v > best[u]) { best[u] = v; arg[u] = i; }
                }
            };
            // LB candidates i0 .. i0+LB-1 from resident rows (slot = row): every
            // read is issued before the first one is used
            auto relax_batch = [&](int i0) __attribute__((always_inline)) {
                FsCand c[LB];
                float m[LB][U];
#pragma unroll
                for (int a = 0; a < LB; ++a) c[a] = cj[i0 + a];
#pragma unroll
                for (int a = 0; a < LB; ++a) {
                    const int lo = rows0 + (i0 + a) * RS * 4;
#pragma unroll
                    for (int u = 0; u < U; ++u) m[a][u] = lds_ld(max(tc4[u] + c[a].off, lo));
                }
#pragma unroll
                for (int a = 0; a < LB; ++a) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const float v = m[a][u] + c[a].imp;
                        if (v > best[u]) { best[u] = v; arg[u] = i0 + a; }
                    }
                }
            };
            // the first batch from global memory is in flight while the resident
            // rows are used; candidates are still taken in ascending i
            if (na < nc) fetch(na);
            int i = 0;
            for (; i + LB <= na; i += LB) relax_batch(i);
            for (; i < na; ++i) relax_lds(i, i);
            for (int i0 = na; i0 < nc; i0 += CH) {
                if (i0 != na) fetch(i0);
                use(i0);
            }
            for (int i2 = nc; i2 < j; ++i2) relax_lds(i2, slot_of(i2));   // at most two rows
            // A row is read back from global memory three rows after it was
            // stored at the earliest.  Waiting here for the stores of the row
            // before (long acknowledged) makes that certain: when a row is
            // read, every wave has passed this point and a barrier since.
            if (j > NR) wait_vm(0);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (t[u] < P) {
                    Mb[(size_t)j * P + t[u]] = best[u];
                    if (STORE_K) Kb[(size_t)j * P + t[u]] = (uint8_t)arg[u];
                    lds_st(rows0 + (slot_of(j) * RS + 1 + t[u]) * 4, best[u]);
                }
        }
        __syncthreads();
    }

    if constexpr (QUERIES) {
        // ---------------- set recovery for the queries of this instance ----------------
        // Every wave has waited for its stores (the tables are complete at the
        // level all compute units share) before any wave reads them back.  The
        // lists of the walks lie over the candidate table, which is done with.
        int32_t (*lists)[2][FS_LIST] = (int32_t (*)[2][FS_LIST])smem;
        wait_vm(0);
        __syncthreads();
        const int nchunks = (qs.Q + 63) / 64;
        for (int c = wave; c < nchunks; c += nw) {
            const int q = c * 64 + lane;
            const int qb = q < qs.Q ? qs.q_inst[q] : -2;
            // a query that names no instance is answered ("bad query") by workgroup 0
            const bool mine = q < qs.Q && (qb == b || (b == 0 && (qb < 0 || qb >= B)));
            unsigned long long todo = __ballot(mine);
            while (todo != 0) {
                const int l = __builtin_ctzll(todo);
                todo &= todo - 1;
                const int qq = c * 64 + l;
                backtrack_query<true>(qq, bt_uniform(qs.q_inst[qq]), bt_uniform(qs.q_T0[qq]), B, L, P,
                                      Topt, split, I, M, STORE_K ? K : nullptr, qs.A, qs.A_len, qs.S,
                                      qs.S_len, qs.obj, qs.lat, qs.status, lists[wave][0],
                                      lists[wave][1], lane);
            }
        }
    }
}

// LDS bytes with `nslots` slots for rows of M (their space also holds the copy
// of T during stage 1)
static size_t fs_lds_bytes(int L, int P, int nslots)
{
    const size_t ld2 = (size_t)(L + 1) * (L + 1);
    // (at least the room the lists of the query phase take, which reuse this block)
    return std::max(ld2 * sizeof(FsCand) + std::max((size_t)nslots * (P + 1) * 4, ld2 * 4),
                    (size_t)FS_LIST_BYTES);
}

// slots that fit, at most one per row
static int fs_slots(int L, int P, int lds_limit)
{
    const size_t cand_bytes = (size_t)(L + 1) * (L + 1) * sizeof(FsCand);
    if ((size_t)lds_limit < cand_bytes) return 0;
    const size_t n = ((size_t)lds_limit - cand_bytes) / ((size_t)(P + 1) * 4);
    return (int)std::min<size_t>(n, (size_t)L + 1);
}

bool fused_small_supported(int L, int P, int lds_limit)
{
    if (L < 1 || L > 63 || P < 1 || P > 2048) return false;
    const int n = fs_slots(L, P, lds_limit);
    // every row resident, or at least one resident row and the shared slots
    return (n == L + 1 || n >= 1 + FS_RING) && fs_lds_bytes(L, P, n) <= (size_t)lds_limit;
}

// Q == 0: stage 1 and stage 2 only; otherwise the queries are answered in the same launch
hipError_t launch_fused_small(int B, int L, int P, const int32_t* T, const float* I, int32_t* Topt,
                              uint8_t* split, float* M, uint8_t* K, int lds_limit, int Q,
                              const int32_t* q_inst, const int32_t* q_T0, int32_t* A, int32_t* A_len,
                              int32_t* S, int32_t* S_len, float* obj, int32_t* lat, int32_t* status,
                              hipStream_t st)
{
    if (!fused_small_supported(L, P, lds_limit)) return hipErrorInvalidValue;
    const int nslots = fs_slots(L, P, lds_limit);
    const int NR = nslots == L + 1 ? nslots : nslots - FS_RING;
    const size_t lds = fs_lds_bytes(L, P, nslots);
    const int U = P > 1024 ? 2 : 1;
    // a thread per column (two when P > 1024), and at least a wave per source row of stage 1
    const int NT = std::min(1024, std::max(((P + U - 1) / U + 63) / 64 * 64, 64 * (L + 1)));
    const FsQueries qs{Q, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status};
    auto go = [&](auto kernel) {
        // (more than 64 KB of dynamic LDS has to be asked for)
        hipError_t e = hipFuncSetAttribute((const void*)kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, dim3(B), dim3(NT), lds, st, B, L, P, NR, T, I, Topt, split, M, K, qs);
        return hipGetLastError();
    };
    if (Q > 0) {
        if (U == 1) return K ? go(fused_small_kernel<1, true, true>) : go(fused_small_kernel<1, false, true>);
        return K ? go(fused_small_kernel<2, true, true>) : go(fused_small_kernel<2, false, true>);
    }
    if (U == 1) return K ? go(fused_small_kernel<1, true, false>) : go(fused_small_kernel<1, false, false>);
    return K ? go(fused_small_kernel<2, true, false>) : go(fused_small_kernel<2, false, false>);
}

}  // namespace dpc
