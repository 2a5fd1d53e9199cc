// C-ABI entry points of libdpc.so: argument checks and kernel launches.
#include "dpc_internal.h"
#include "dpc_hooks.h"

namespace {

int num_compute_units()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            n <= 0)
            return -1;
        cached[dev] = n;
    }
    return cached[dev];
}

// LDS bytes one workgroup may use on the current device
int lds_per_workgroup()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
            n <= 0)
            return -1;
        cached[dev] = n;
    }
    return cached[dev];
}

bool shape_ok(int B, int L, int P)
{
    return B >= 1 && L >= 1 && L <= DPC_MAX_L && P >= 1 &&
           (int64_t)B * (L + 1) * (int64_t)P < ((int64_t)1 << 40);
}

// layout of the extended solver's workspace: the two virtual tables, then the
// stage-2 workspace of the chain of 2L+2 virtual layers
struct ExtLayout { size_t tv_off, iv_off, s2_off, total; };
ExtLayout ext_layout(int B, int L, int P)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t V = 2 * (size_t)L + 3;
    ExtLayout l;
    l.tv_off = 0;
    l.iv_off = up(4 * (size_t)B * V * V);
    l.s2_off = l.iv_off + up(4 * (size_t)B * V * V);
    l.total = l.s2_off + dpc::stage2_workspace_bytes(B, 2 * L + 2, P);
    return l;
}

bool ext_shape_ok(int B, int L, int P) { return L >= 1 && L <= DPC_EXT_MAX_L && shape_ok(B, 2 * L + 2, P); }

}  // namespace

namespace dpc {

bool stage2_runs_row_by_row(int P, int shape)
{
    return shape == DPC_SHAPE_ROWS || P < 16 || P >= (1 << 29);
}

int stage2_run(int B, int L, int P, ToptRef Topt, const float* I, float* M, uint8_t* K,
               void* workspace, int shape, hipStream_t stream)
{
    hipError_t e;
    // The wave-window family copies whole 16-byte cells of a row and keeps byte
    // offsets inside a row in 32 bits: tables narrower than 16 budgets (and
    // absurdly wide ones) are solved row by row, one launch per row.
    if (stage2_runs_row_by_row(P, shape)) {
        // this family uses no workspace; clear the header so that a later
        // dpc_stage2_check reads "no error"
        e = launch_clear_words(workspace, S2_HEADER_WORDS, stream);
        if (e == hipSuccess) e = launch_stage2_rows(B, L, P, Topt, I, M, K, stream);
    } else {
        const int ncu = num_compute_units();
        if (ncu <= 0) return DPC_ERR_HIP;
        e = launch_stage2_wave(B, L, P, Topt, I, M, K, workspace, ncu,
                               shape == 0 ? 0 : shape - DPC_SHAPE_WAVE_BASE, stream);
    }
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

}  // namespace dpc

extern "C" {

const char* dpc_status_string(int code)
{
    switch (code) {
        case DPC_OK: return "DPC_OK";
        case DPC_ERR_NULL: return "DPC_ERR_NULL: a required pointer is NULL";
        case DPC_ERR_SHAPE: return "DPC_ERR_SHAPE: B, L, P or Q outside the supported range";
        case DPC_ERR_WORKSPACE: return "DPC_ERR_WORKSPACE: workspace too small or misaligned";
        case DPC_ERR_HIP: return "DPC_ERR_HIP: a HIP runtime call failed";
        case DPC_ERR_TIMEOUT: return "DPC_ERR_TIMEOUT: a bounded in-kernel wait ran out";
        default: return "unknown libdpc status";
    }
}

int dpc_stage1_minplus(int32_t B, int32_t L, const int32_t* T, int32_t* Topt, uint8_t* split,
                       void* stream)
{
    if (!T || !Topt || !split) return DPC_ERR_NULL;
    if (!shape_ok(B, L, 1)) return DPC_ERR_SHAPE;
    hipError_t e = dpc::launch_stage1(B, L, T, Topt, split, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

size_t dpc_stage2_workspace_bytes(int32_t B, int32_t L, int32_t P)
{
    if (!shape_ok(B, L, P)) return 0;
    return dpc::stage2_workspace_bytes(B, L, P);
}

int dpc_stage2_knapsack(int32_t B, int32_t L, int32_t P, const int32_t* Topt, const float* I,
                        float* M, uint8_t* K, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    if (!Topt || !I || !M || !workspace) return DPC_ERR_NULL;
    if (!shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    if (workspace_bytes < dpc_stage2_workspace_bytes(B, L, P) || ((uintptr_t)workspace & 255))
        return DPC_ERR_WORKSPACE;
    return dpc::stage2_run(B, L, P, dpc::ToptRef{Topt, 1}, I, M, K, workspace, 0, (hipStream_t)stream);
}

int dpc_stage2_knapsack_shared(int32_t B, int32_t L, int32_t P, int32_t share, const int32_t* Topt,
                               const float* I, float* M, uint8_t* K, void* workspace,
                               size_t workspace_bytes, void* stream)
{
    if (!Topt || !I || !M || !workspace) return DPC_ERR_NULL;
    if (!shape_ok(B, L, P) || share < 1) return DPC_ERR_SHAPE;
    if (workspace_bytes < dpc_stage2_workspace_bytes(B, L, P) || ((uintptr_t)workspace & 255))
        return DPC_ERR_WORKSPACE;
    return dpc::stage2_run(B, L, P, dpc::ToptRef{Topt, share}, I, M, K, workspace, 0, (hipStream_t)stream);
}

int dpc_stage2_knapsack_shape(int32_t B, int32_t L, int32_t P, const int32_t* Topt, const float* I,
                              float* M, uint8_t* K, void* workspace, size_t workspace_bytes,
                              int32_t shape, void* stream)
{
    if (!Topt || !I || !M || !workspace) return DPC_ERR_NULL;
    if (!shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    if (shape != 0 && shape != DPC_SHAPE_ROWS &&
        !dpc::stage2_wave_shape_known(shape - DPC_SHAPE_WAVE_BASE))
        return DPC_ERR_SHAPE;
    if (workspace_bytes < dpc_stage2_workspace_bytes(B, L, P) || ((uintptr_t)workspace & 255))
        return DPC_ERR_WORKSPACE;
    return dpc::stage2_run(B, L, P, dpc::ToptRef{Topt, 1}, I, M, K, workspace, shape, (hipStream_t)stream);
}

int dpc_stage2_check(const void* workspace, void* stream)
{
    if (!workspace) return DPC_ERR_NULL;
    uint32_t word = 0;
    if (hipMemcpyAsync(&word, (const char*)workspace + dpc::S2_ERROR_WORD_OFFSET, sizeof(word),
                       hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return DPC_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DPC_ERR_HIP;
    return word != 0 ? DPC_ERR_TIMEOUT : DPC_OK;
}

namespace {
int backtrack_checked(int32_t B, int32_t L, int32_t P, int32_t share, const int32_t* Topt,
                      const uint8_t* split, const float* I, const float* M, const uint8_t* K, int32_t Q,
                      const int32_t* q_inst, const int32_t* q_T0, int32_t* A, int32_t* A_len,
                      int32_t* S, int32_t* S_len, float* obj, int32_t* lat, int32_t* status,
                      void* stream)
{
    if (Q < 0 || share < 1) return DPC_ERR_SHAPE;
    if (!shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    if (Q == 0) return DPC_OK;
    if (!Topt || !split || !I || !M || !q_inst || !q_T0 || !A || !A_len || !S || !S_len || !obj ||
        !lat || !status)
        return DPC_ERR_NULL;
    hipError_t e = dpc::launch_backtrack(B, L, P, Topt, split, I, M, K, Q, q_inst, q_T0, A, A_len,
                                         S, S_len, obj, lat, status, share, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}
}  // namespace

int dpc_backtrack(int32_t B, int32_t L, int32_t P, const int32_t* Topt, const uint8_t* split,
                  const float* I, const float* M, const uint8_t* K, int32_t Q,
                  const int32_t* q_inst, const int32_t* q_T0, int32_t* A, int32_t* A_len,
                  int32_t* S, int32_t* S_len, float* obj, int32_t* lat, int32_t* status,
                  void* stream)
{
    return backtrack_checked(B, L, P, 1, Topt, split, I, M, K, Q, q_inst, q_T0, A, A_len, S, S_len,
                             obj, lat, status, stream);
}

int dpc_backtrack_shared(int32_t B, int32_t L, int32_t P, int32_t share, const int32_t* Topt,
                         const uint8_t* split, const float* I, const float* M, const uint8_t* K,
                         int32_t Q, const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                         int32_t* A_len, int32_t* S, int32_t* S_len, float* obj, int32_t* lat,
                         int32_t* status, void* stream)
{
    return backtrack_checked(B, L, P, share, Topt, split, I, M, K, Q, q_inst, q_T0, A, A_len, S,
                             S_len, obj, lat, status, stream);
}

int dpc_ext_importance_maxplus(int32_t B, int32_t L, const float* I4, float* Iopt, uint8_t* bsplit,
                               void* stream)
{
    if (!I4 || !Iopt || !bsplit) return DPC_ERR_NULL;
    if (!shape_ok(B, L, 1)) return DPC_ERR_SHAPE;
    hipError_t e = dpc::launch_ext_iopt(B, L, I4, Iopt, bsplit, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

size_t dpc_ext_workspace_bytes(int32_t B, int32_t L, int32_t P)
{
    if (!ext_shape_ok(B, L, P)) return 0;
    return ext_layout(B, L, P).total;
}

int dpc_ext_knapsack(int32_t B, int32_t L, int32_t P, const int32_t* Topt, const float* Iopt,
                     float* D, uint8_t* Kx, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!Topt || !Iopt || !D || !workspace) return DPC_ERR_NULL;
    if (!ext_shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    if (workspace_bytes < dpc_ext_workspace_bytes(B, L, P) || ((uintptr_t)workspace & 255))
        return DPC_ERR_WORKSPACE;
    const ExtLayout lay = ext_layout(B, L, P);
    char* base = (char*)workspace;
    int32_t* Tv = (int32_t*)(base + lay.tv_off);
    float* Iv = (float*)(base + lay.iv_off);
    // The wave-window family computes the entries of the virtual tables where it
    // reads them (its preparation kernel and the pair settlement); the
    // row-by-row family reads expanded tables.
    if (!dpc::stage2_runs_row_by_row(P, 0))
        return dpc::stage2_run(B, 2 * L + 2, P, dpc::ToptRef{Topt, 1, L, Iopt}, nullptr, D, Kx,
                               base + lay.s2_off, 0, (hipStream_t)stream);
    hipError_t e = dpc::launch_ext_expand(B, L, Topt, Iopt, Tv, Iv, (hipStream_t)stream);
    if (e != hipSuccess) return DPC_ERR_HIP;
    return dpc::stage2_run(B, 2 * L + 2, P, dpc::ToptRef{Tv, 1}, Iv, D, Kx, base + lay.s2_off, 0,
                           (hipStream_t)stream);
}

int dpc_ext_check(int32_t B, int32_t L, int32_t P, const void* workspace, void* stream)
{
    if (!workspace) return DPC_ERR_NULL;
    if (!ext_shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    return dpc_stage2_check((const char*)workspace + ext_layout(B, L, P).s2_off, stream);
}

int dpc_ext_backtrack(int32_t B, int32_t L, int32_t P, const int32_t* Topt, const uint8_t* split,
                      const uint8_t* bsplit, const float* D, const uint8_t* Kx, int32_t Q,
                      const int32_t* q_inst, const int32_t* q_T0, int32_t* A, int32_t* A_len,
                      int32_t* S, int32_t* S_len, int32_t* Bs, int32_t* B_len, float* obj,
                      int32_t* lat, int32_t* a_last, int32_t* status, void* stream)
{
    if (Q < 0) return DPC_ERR_SHAPE;
    if (!ext_shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    if (Q == 0) return DPC_OK;
    if (!Topt || !split || !bsplit || !D || !Kx || !q_inst || !q_T0 || !A || !A_len || !S ||
        !S_len || !Bs || !B_len || !obj || !lat || !a_last || !status)
        return DPC_ERR_NULL;
    hipError_t e = dpc::launch_ext_backtrack(B, L, P, Topt, split, bsplit, D, Kx, Q, q_inst, q_T0,
                                             A, A_len, S, S_len, Bs, B_len, obj, lat, a_last,
                                             status, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_stage12_fused_supported(int32_t L, int32_t P)
{
    const int lds = lds_per_workgroup();
    return lds > 0 && dpc::fused_small_supported(L, P, lds) ? 1 : 0;
}

int dpc_stage12_fused(int32_t B, int32_t L, int32_t P, const int32_t* T, const float* I,
                      int32_t* Topt, uint8_t* split, float* M, uint8_t* K, void* stream)
{
    if (!T || !I || !Topt || !split || !M) return DPC_ERR_NULL;
    if (!shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    const int lds = lds_per_workgroup();
    if (lds <= 0) return DPC_ERR_HIP;
    if (!dpc::fused_small_supported(L, P, lds)) return DPC_ERR_SHAPE;
    hipError_t e = dpc::launch_fused_small(B, L, P, T, I, Topt, split, M, K, lds, 0, nullptr, nullptr,
                                           nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                           nullptr, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_solve_fused(int32_t B, int32_t L, int32_t P, const int32_t* T, const float* I, int32_t* Topt,
                    uint8_t* split, float* M, uint8_t* K, int32_t Q, const int32_t* q_inst,
                    const int32_t* q_T0, int32_t* A, int32_t* A_len, int32_t* S, int32_t* S_len,
                    float* obj, int32_t* lat, int32_t* status, void* stream)
{
    if (Q < 0) return DPC_ERR_SHAPE;
    if (!T || !I || !Topt || !split || !M) return DPC_ERR_NULL;
    if (Q > 0 && (!q_inst || !q_T0 || !A || !A_len || !S || !S_len || !obj || !lat || !status))
        return DPC_ERR_NULL;
    if (!shape_ok(B, L, P)) return DPC_ERR_SHAPE;
    const int lds = lds_per_workgroup();
    if (lds <= 0) return DPC_ERR_HIP;
    if (!dpc::fused_small_supported(L, P, lds)) return DPC_ERR_SHAPE;
    hipError_t e = dpc::launch_fused_small(B, L, P, T, I, Topt, split, M, K, lds, Q, q_inst, q_T0, A,
                                           A_len, S, S_len, obj, lat, status, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_importance_shift(int32_t B, int32_t L, int32_t F, int32_t n_alpha, const float* I_raw,
                         const float* alpha, float* I_out, double* mean_out, void* stream)
{
    if (!shape_ok(B, L, 1) || (F != 1 && F != 4) || n_alpha < 0 || n_alpha > 65535)
        return DPC_ERR_SHAPE;
    if (n_alpha == 0) return DPC_OK;
    if (!I_raw || !alpha || !I_out) return DPC_ERR_NULL;
    hipError_t e = dpc::launch_importance_shift(B, L, F, n_alpha, I_raw, alpha, I_out, mean_out,
                                                (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_front(int32_t B, int32_t L, int32_t P, const float* M, int32_t cap, int32_t* front_t,
              float* front_obj, int32_t* front_len, void* stream)
{
    if (!shape_ok(B, L, P) || cap < 0) return DPC_ERR_SHAPE;
    if (!M || !front_len || (cap > 0 && (!front_t || !front_obj))) return DPC_ERR_NULL;
    hipError_t e = dpc::launch_front(B, L, P, M, cap, front_t, front_obj, front_len,
                                     (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_front_queries(int32_t B, int32_t cap, const int32_t* front_t, const int32_t* front_len,
                      int32_t qcap, int32_t* q_inst, int32_t* q_T0, int32_t* q_count, void* stream)
{
    if (B < 1 || B > 65535 * 1024 || cap < 0 || qcap < 0) return DPC_ERR_SHAPE;
    if (!front_len || !q_count || (cap > 0 && !front_t) || (qcap > 0 && (!q_inst || !q_T0)))
        return DPC_ERR_NULL;
    hipError_t e = dpc::launch_front_queries(B, cap, front_t, front_len, qcap, q_inst, q_T0,
                                             q_count, (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

int dpc_chain_latency(int32_t B, int32_t L, const int32_t* T, int32_t Q, const int32_t* q_inst,
                      const int32_t* X, const int32_t* X_len, int32_t* lat, void* stream)
{
    if (Q < 0 || !shape_ok(B, L, 1)) return DPC_ERR_SHAPE;
    if (Q == 0) return DPC_OK;
    if (!T || !q_inst || !X || !X_len || !lat) return DPC_ERR_NULL;
    hipError_t e = dpc::launch_chain_latency(B, L, T, Q, q_inst, X, X_len, lat,
                                             (hipStream_t)stream);
    return e == hipSuccess ? DPC_OK : DPC_ERR_HIP;
}

}  // extern "C"
