// CPU emulation of dpc_solve_fused's kernel (see hip/hip_runtime.h in this
// folder): compiled for the host, unchanged, and run one workgroup at a time
// under AddressSanitizer.  Usage: emu_fused <in.bin> <out.bin>
//   in : int32 B, L, P, lds_limit (dynamic LDS a workgroup may use), Q;
//        int32 T[B][L+1][L+1];  float I[B][L+1][L+1];  int32 q_inst[Q];  int32 q_T0[Q]
//   out: int32 Topt[B][L+1][L+1];  uint8 split[B][L+1][L+1];  float M[B][L+1][P];  uint8 K[B][L+1][P];
//        int32 A[Q][L], S[Q][L], A_len[Q], S_len[Q], lat[Q], status[Q];  float obj[Q]
#define DPC_HOST_EMU 1
#include "../../paper_2301_12187_amd/csrc/fused_small.hip"

int main(int argc, char** argv)
{
    if (argc != 3) return 2;
    FILE* f = std::fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[5];
    if (std::fread(hd, 4, 5, f) != 5) return 2;
    const int B = hd[0], L = hd[1], P = hd[2], lds_limit = hd[3], Q = hd[4], ld = L + 1;
    const size_t n2 = (size_t)B * ld * ld, cells = (size_t)B * ld * P;
    // exact-size heap blocks: the sanitizer's red zones sit right behind them
    int32_t* T = (int32_t*)std::malloc(n2 * 4);
    float* I = (float*)std::malloc(n2 * 4);
    if (std::fread(T, 4, n2, f) != n2) return 2;
    if (std::fread(I, 4, n2, f) != n2) return 2;
    int32_t* qi = (int32_t*)std::malloc((size_t)Q * 4 + 4);
    int32_t* qt = (int32_t*)std::malloc((size_t)Q * 4 + 4);
    if (std::fread(qi, 4, Q, f) != (size_t)Q) return 2;
    if (std::fread(qt, 4, Q, f) != (size_t)Q) return 2;
    std::fclose(f);
    int32_t* A = (int32_t*)std::malloc((size_t)Q * L * 4 + 4);
    int32_t* S = (int32_t*)std::malloc((size_t)Q * L * 4 + 4);
    int32_t* small = (int32_t*)std::malloc((size_t)Q * 4 * 4 + 4);   // A_len, S_len, lat, status
    float* obj = (float*)std::malloc((size_t)Q * 4 + 4);
    for (size_t x = 0; x < (size_t)Q * L; ++x) A[x] = S[x] = -9;
    int32_t* Topt = (int32_t*)std::malloc(n2 * 4);
    uint8_t* split = (uint8_t*)std::malloc(n2);
    float* M = (float*)std::malloc(cells * 4);
    uint8_t* K = (uint8_t*)std::malloc(cells);
    for (size_t x = 0; x < n2; ++x) { Topt[x] = -7; split[x] = 0xEE; }
    for (size_t x = 0; x < cells; ++x) { M[x] = NAN; K[x] = 0xEE; }
    const hipError_t e = dpc::launch_fused_small(B, L, P, T, I, Topt, split, M, K, lds_limit, Q, qi, qt, A,
                                                 small, S, small + Q, obj, small + 2 * Q, small + 3 * Q,
                                                 nullptr);
    if (e != hipSuccess) { std::fprintf(stderr, "launch failed\n"); return 3; }
    f = std::fopen(argv[2], "wb");
    std::fwrite(Topt, 4, n2, f);
    std::fwrite(split, 1, n2, f);
    std::fwrite(M, 4, cells, f);
    std::fwrite(K, 1, cells, f);
    std::fwrite(A, 4, (size_t)Q * L, f);
    std::fwrite(S, 4, (size_t)Q * L, f);
    std::fwrite(small, 4, (size_t)Q * 4, f);
    std::fwrite(obj, 4, Q, f);
    std::fclose(f);
    std::free(qi); std::free(qt); std::free(A); std::free(S); std::free(small); std::free(obj);
    std::free(T); std::free(I); std::free(Topt); std::free(split); std::free(M); std::free(K);
    return 0;
}
