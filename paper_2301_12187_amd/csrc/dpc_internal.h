// Internal declarations shared by the translation units of libdpc.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "dpc.h"

namespace dpc {

// Index of I4[k][l][a][b] / Iopt[k][l][a][b] of the extended solver inside an instance
__host__ __device__ __forceinline__ size_t i4_index(int ld, int k, int l, int a, int b)
{
    return ((((size_t)k * ld + l) * 2 + a) * 2 + b);
}

// The latency tables of a batch as stage 2 reads them: instance b uses table
// b / share.  share > 1: consecutive instances are copies of one network with
// different importances (a sweep over the normalisation constant) and share
// the one table stage 1 computed for it.
// ext_L > 0: the chain stage 2 runs on is the extended solver's chain of
// (layer, flag) states over ext_L real layers (Algorithm 4 as Algorithm 2 on the
// virtual layers v = 2 l + a, plus a last one); `base` is then the real Topt
// and ext_iopt the real I_opt, and the kernels that can (operands()) compute
// the virtual entries from them instead of reading expanded tables.
struct ToptRef {
    const int32_t* base;
    int share;
    int ext_L = 0;
    const float* ext_iopt = nullptr;
    __host__ __device__ const int32_t* of(int b, int ld) const
    {
        return base + (size_t)(share > 1 ? b / share : b) * ld * ld;
    }
    // latency and importance of the block (i, j) of instance b of a chain whose
    // tables have ld = (layers + 1) rows; I: the importances of a plain chain
    __device__ __forceinline__ void operands(const float* __restrict__ I, int b, int ld, int i, int j,
                                              int32_t& t, float& imp) const
    {
        if (ext_L == 0) {
            t = of(b, ld)[(size_t)i * ld + j];
            imp = I[((size_t)b * ld + i) * ld + j];
            return;
        }
        // An entry (u, v) = (i, j), u < v, of the virtual chain, V = 2 L + 3 layers:
        //   u = 0, v = 1      latency 0, importance +0  (D[0][t][1] = D[0][t][0] = +0)
        //   v <= 2L+1         from (k', alpha') = (u / 2, u % 2) to (l, a) = (v / 2, v % 2), k' < l:
        //                     latency Topt[k'][l], importance I_opt[k'][l][alpha'][a]
        //   v = 2L+2          from (L, 0) and (L, 1): latency 0, importance +0
        // everything else: none (latency DPC_INF, importance -inf).
        const int L = ext_L, rl = L + 1, V = 2 * L + 3;
        t = DPC_INF;
        imp = -INFINITY;
        if (i < j) {
            const int kp = i >> 1, al = i & 1, l = j >> 1, a = j & 1;
            if (j == V - 1) {
                if (kp == L) { t = 0; imp = 0.0f; }
            } else if (kp < l) {
                t = base[(size_t)b * rl * rl + (size_t)kp * rl + l];
                imp = ext_iopt[(size_t)b * rl * rl * 4 + i4_index(rl, kp, l, al, a)];
            } else if (i == 0 && j == 1) {
                t = 0;
                imp = 0.0f;
            }
        }
    }
};

// kernel launchers; each returns a hipError_t from the launch
hipError_t launch_stage1(int B, int L, const int32_t* T, int32_t* Topt, uint8_t* split,
                         hipStream_t st);
hipError_t launch_stage2_rows(int B, int L, int P, ToptRef Topt, const float* I,
                              float* M, uint8_t* K, hipStream_t st);
// zero `nwords` 32-bit words with a small kernel (safe to record into a HIP graph)
hipError_t launch_clear_words(void* p, int nwords, hipStream_t st);
size_t stage2_workspace_bytes(int B, int L, int P);
// byte offset, in a stage-2 workspace, of the word a kernel sets when a bounded wait ran out
constexpr size_t S2_ERROR_WORD_OFFSET = 148;
constexpr int S2_HEADER_WORDS = 64;
// shape 0: task shape chosen from the problem size; otherwise a fixed one
// (stage2_wave_shape_known), for tests and measurements
hipError_t launch_stage2_wave(int B, int L, int P, ToptRef Topt, const float* I, float* M,
                              uint8_t* K, void* workspace, int num_cu, int shape, hipStream_t st);
bool stage2_wave_shape_known(int shape);
// Stage 2 on checked arguments with the kernel family `shape` selects (see
// dpc_hooks.h; 0 = the default choice).  Returns a DPC_* code.
int stage2_run(int B, int L, int P, ToptRef Topt, const float* I, float* M, uint8_t* K,
               void* workspace, int shape, hipStream_t st);
// whether stage2_run takes the one-launch-per-row family for this width and shape
bool stage2_runs_row_by_row(int P, int shape);
hipError_t launch_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                            const float* I, const float* M, const uint8_t* K, int Q,
                            const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                            int32_t* A_len, int32_t* S, int32_t* S_len, float* obj,
                            int32_t* lat, int32_t* status, int share, hipStream_t st);

// extended solver (Appendix B): Algorithm 3, the virtual tables of Algorithm 4, set recovery
hipError_t launch_ext_iopt(int B, int L, const float* I4, float* Iopt, uint8_t* bsplit,
                           hipStream_t st);
hipError_t launch_ext_expand(int B, int L, const int32_t* Topt, const float* Iopt, int32_t* Tv,
                             float* Iv, hipStream_t st);
hipError_t launch_ext_backtrack(int B, int L, int P, const int32_t* Topt, const uint8_t* split,
                                const uint8_t* bsplit, const float* D, const uint8_t* Kx, int Q,
                                const int32_t* q_inst, const int32_t* q_T0, int32_t* A,
                                int32_t* A_len, int32_t* S, int32_t* S_len, int32_t* Bs,
                                int32_t* B_len, float* obj, int32_t* lat, int32_t* a_last,
                                int32_t* status, hipStream_t st);

// stage 1 + stage 2 in one launch for small instances; lds_limit = LDS bytes a workgroup may use
bool fused_small_supported(int L, int P, int lds_limit);
// Q > 0: the queries are answered in the same launch (each by the workgroup of its instance)
hipError_t launch_fused_small(int B, int L, int P, const int32_t* T, const float* I, int32_t* Topt,
                              uint8_t* split, float* M, uint8_t* K, int lds_limit, int Q,
                              const int32_t* q_inst, const int32_t* q_T0, int32_t* A, int32_t* A_len,
                              int32_t* S, int32_t* S_len, float* obj, int32_t* lat, int32_t* status,
                              hipStream_t st);

// sweep steps: importance normalisation, trade-off curve, latency of a given merge set
hipError_t launch_importance_shift(int B, int L, int F, int n_alpha, const float* I_raw,
                                   const float* alpha, float* I_out, double* mean_out,
                                   hipStream_t st);
hipError_t launch_front(int B, int L, int P, const float* M, int cap, int32_t* front_t,
                        float* front_obj, int32_t* front_len, hipStream_t st);
hipError_t launch_front_queries(int B, int cap, const int32_t* front_t, const int32_t* front_len,
                                int qcap, int32_t* q_inst, int32_t* q_T0, int32_t* q_count,
                                hipStream_t st);
hipError_t launch_chain_latency(int B, int L, const int32_t* T, int Q, const int32_t* q_inst,
                                const int32_t* X, const int32_t* X_len, int32_t* lat,
                                hipStream_t st);

}  // namespace dpc
