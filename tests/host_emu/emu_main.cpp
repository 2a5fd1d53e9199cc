// CPU emulation of dpc_stage2_knapsack's wave-window kernel family (see
// hip/hip_runtime.h in this folder): the preparation kernels and the main
// kernel are compiled for the host, unchanged, and run one workgroup at a
// time under AddressSanitizer.  Usage: emu <in.bin> <out.bin>
//   in : int32 B, L, P, shape;  int32 Topt[B][L+1][L+1];  float I[B][L+1][L+1]
//   out: float M[B][L+1][P];  uint8 K[B][L+1][P]
#define DPC_HOST_EMU 1
#include "../../paper_2301_12187_amd/csrc/stage2_pack.hip"
#include "../../paper_2301_12187_amd/csrc/stage2_wave.hip"

int main(int argc, char** argv)
{
    if (argc != 3) return 2;
    FILE* f = std::fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[4];
    if (std::fread(hd, 4, 4, f) != 4) return 2;
    const int B = hd[0], L = hd[1], P = hd[2], shape = hd[3], ld = L + 1;
    std::vector<int32_t> Topt((size_t)B * ld * ld);
    std::vector<float> I((size_t)B * ld * ld);
    if (std::fread(Topt.data(), 4, Topt.size(), f) != Topt.size()) return 2;
    if (std::fread(I.data(), 4, I.size(), f) != I.size()) return 2;
    std::fclose(f);
    const size_t cells = (size_t)B * ld * P;
    // exact-size heap blocks: the sanitizer's red zones sit right behind them
    float* M = (float*)std::malloc(cells * 4);
    uint8_t* K = (uint8_t*)std::malloc(cells);
    for (size_t x = 0; x < cells; ++x) { M[x] = NAN; K[x] = 0xEE; }
    const size_t wsb = dpc::stage2_workspace_bytes(B, L, P);
    char* ws = (char*)std::aligned_alloc(256, wsb);
    std::memset(ws, 0xA5, wsb);
    emu::register_region(M, cells * 4, "M");
    emu::register_region(ws, wsb, "workspace");
    emu::g_lds_lo = nullptr;
    emu::g_lds_hi = (const char*)~(uintptr_t)0;
    const hipError_t e = dpc::launch_stage2_wave(B, L, P, dpc::ToptRef{Topt.data(), 1}, I.data(), M, K, ws, 1, shape, nullptr);
    if (e != hipSuccess) { std::fprintf(stderr, "launch failed\n"); return 3; }
    if (std::getenv("EMU_DUMP_HEADER")) { for (int x = 0; x < 40; ++x) std::fprintf(stderr, "%08x ", ((uint32_t*)ws)[x]); std::fprintf(stderr, "\n"); }
    if (((uint32_t*)ws)[dpc::S2_ERROR_WORD_OFFSET / 4] != 0) { std::fprintf(stderr, "error word set\n"); return 4; }
    f = std::fopen(argv[2], "wb");
    std::fwrite(M, 4, cells, f);
    std::fwrite(K, 1, cells, f);
    std::fclose(f);
    std::free(M); std::free(K); std::free(ws);
    return 0;
}
