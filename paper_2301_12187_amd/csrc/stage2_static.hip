// dpc_stage2_knapsack_static: stage 2 (Algorithm 2 / recurrence Eq. 7 of the
// paper) for callers that cannot allocate device memory and have no workspace
// to pass.  The task table, completion counters and repacked operands that
// dpc_stage2_knapsack keeps in the caller's workspace live in a fixed array in
// device memory that belongs to the library; everything else (argument checks,
// kernels, results) is dpc_stage2_knapsack's.
#include <mutex>
#include "dpc_internal.h"

namespace {

// One copy per GPU, held from the moment the code object is loaded on that GPU
// until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address of each GPU's copy is looked up once
// and kept in g_scratch_ptr, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[DPC_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};
std::mutex g_scratch_mutex;

// device address of the current device's copy of `scratch`
int scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return DPC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr)
            return DPC_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DPC_OK;
}

}  // namespace

extern "C" int dpc_stage2_knapsack_static(int32_t B, int32_t L, int32_t P, const int32_t* Topt,
                                          const float* I, float* M, uint8_t* K, void* stream)
{
    if (!Topt || !I || !M) return DPC_ERR_NULL;
    const size_t need = dpc_stage2_workspace_bytes(B, L, P);
    if (need == 0) return DPC_ERR_SHAPE;                    // (B, L or P out of range)
    if (need > (size_t)DPC_STATIC_WORKSPACE_BYTES) return DPC_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != DPC_OK) return rc;
    // the preparation kernels clear the header and the counters they use, so
    // what the previous call left in the array does not matter
    return dpc::stage2_run(B, L, P, dpc::ToptRef{Topt, 1}, I, M, K, ws, 0, (hipStream_t)stream);
}
