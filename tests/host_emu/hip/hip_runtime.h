// Host stand-in for <hip/hip_runtime.h>, used only by the CPU emulation build
// of the stage-2 kernels (tests/host_emu): one workgroup at a time, one host
// thread per lane, a real barrier for __syncthreads.  Every global -> LDS copy
// is checked against the registered buffers, and the build runs under
// AddressSanitizer, so an out-of-bounds index in the kernels' arithmetic
// fails here, on the CPU, instead of on a GPU.
#pragma once
#include <algorithm>
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <type_traits>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __shared__ static
#define address_space(n) unused

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
typedef void* hipStream_t;
inline hipError_t hipGetLastError() { return hipSuccess; }
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }

namespace emu {

struct Barrier {                       // reusable barrier for the threads of one workgroup
    std::mutex m;
    std::condition_variable cv;
    int n = 0, waiting = 0;
    unsigned long gen = 0;
    void wait()
    {
        std::unique_lock<std::mutex> lk(m);
        const unsigned long g = gen;
        if (++waiting == n) { waiting = 0; ++gen; cv.notify_all(); }
        else cv.wait(lk, [&] { return gen != g; });
    }
};
inline Barrier g_barrier;
inline Barrier g_wave_barrier[16];     // the lanes of a wave run in lockstep on the GPU
inline thread_local dim3 t_threadIdx, t_blockIdx, t_blockDim, t_gridDim;
inline int g_exchange[1024];

struct Region { const char* lo; const char* hi; const char* name; };
inline std::vector<Region> g_regions;   // buffers a kernel may read with a global -> LDS copy
inline void register_region(const void* p, size_t bytes, const char* name)
{
    g_regions.push_back({(const char*)p, (const char*)p + bytes, name});
}
inline void check_global(const void* p, size_t n, const char* what)
{
    for (const Region& r : g_regions)
        if ((const char*)p >= r.lo && (const char*)p + n <= r.hi) return;
    std::fprintf(stderr, "EMU: %s of %zu bytes at %p is outside every registered buffer\n", what, n, p);
    std::abort();
}
inline char* g_dyn_lds = nullptr;         // stand-in for the dynamic LDS of the running launch
inline const char* g_lds_lo = nullptr;
inline const char* g_lds_hi = nullptr;

// runs the blocks of a grid one after the other, the threads of a block
// concurrently; the host threads are created once per launch and walk the
// blocks together (a barrier between two blocks: they share the static
// stand-ins of the kernel's LDS arrays)
template <class F>
void launch(dim3 grid, dim3 block, F&& body)
{
    const int nt = (int)block.x;
    g_barrier.n = nt;
    for (int w = 0; w < 16; ++w) g_wave_barrier[w].n = std::min(64, nt);
    std::vector<std::thread> th;
    th.reserve(nt);
    for (int t = 0; t < nt; ++t)
        th.emplace_back([&, t] {
            for (unsigned by = 0; by < grid.y; ++by)
                for (unsigned bx = 0; bx < grid.x; ++bx) {
                    t_threadIdx = dim3(t);
                    t_blockIdx = dim3(bx, by);
                    t_blockDim = block;
                    t_gridDim = grid;
                    body();
                    g_barrier.wait();
                }
        });
    for (auto& x : th) x.join();
}

}  // namespace emu

#define threadIdx emu::t_threadIdx
#define blockIdx emu::t_blockIdx
#define blockDim emu::t_blockDim
#define gridDim emu::t_gridDim
// (the dynamic LDS is an exact-size heap block: the sanitizer sees an access past its end)
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...)                \
    do {                                                                           \
        emu::g_dyn_lds = (size_t)(shmem) ? (char*)std::malloc((size_t)(shmem)) : nullptr; \
        emu::launch(grid, block, [&] { kernel(__VA_ARGS__); });                    \
        std::free(emu::g_dyn_lds);                                                 \
        emu::g_dyn_lds = nullptr;                                                  \
    } while (0)

inline void __syncthreads() { emu::g_barrier.wait(); }
inline void wave_sync() { emu::g_wave_barrier[((int)threadIdx.x >> 6) & 15].wait(); }
template <class T> inline T __builtin_amdgcn_readfirstlane(T v) { return v; }
inline void __builtin_amdgcn_s_sleep(int) { std::this_thread::yield(); }
// (only used to wait for global -> LDS copies, which are synchronous here: what is
//  left of the wait is that every lane of the wave has made its copy)
inline void __builtin_amdgcn_s_waitcnt(int) { wave_sync(); }
inline long long wall_clock64() { return 0; }

inline unsigned __umul24(unsigned a, unsigned b) { return (a & 0xFFFFFFu) * (b & 0xFFFFFFu); }
inline int min(int a, int b) { return a < b ? a : b; }
inline int max(int a, int b) { return a > b ? a : b; }
inline unsigned min(unsigned a, unsigned b) { return a < b ? a : b; }
inline unsigned max(unsigned a, unsigned b) { return a > b ? a : b; }

#define __HIP_MEMORY_SCOPE_AGENT 0
template <class T> inline T __hip_atomic_load(const T* p, int order, int) { T v; __atomic_load(p, &v, order); return v; }
template <class T> inline void __hip_atomic_store(T* p, T v, int order, int) { __atomic_store(p, &v, order); }
template <class T> inline T __hip_atomic_fetch_add(T* p, T v, int order, int) { return __atomic_fetch_add(p, v, order); }
inline unsigned atomicAdd(unsigned* p, unsigned v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
inline int atomicAdd(int* p, int v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
inline int atomicMax(int* p, int v)
{
    int old = __atomic_load_n(p, __ATOMIC_RELAXED);
    while (old < v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) {}
    return old;
}

// value of lane (lane - d) of the same 64-lane wave; every lane of the wave calls it
inline int __shfl_up(int v, int d, int)
{
    const int t = (int)threadIdx.x;
    emu::g_exchange[t] = v;
    wave_sync();
    const int r = (t & 63) >= d ? emu::g_exchange[t - d] : v;
    wave_sync();
    return r;
}

// value of lane `src` of the same wave; every lane of the wave calls it
inline int __shfl(int v, int src, int)
{
    const int t = (int)threadIdx.x;
    emu::g_exchange[t] = v;
    wave_sync();
    const int r = emu::g_exchange[(t & ~63) + (src & 63)];
    wave_sync();
    return r;
}

inline int __builtin_amdgcn_readlane(int v, int src) { return __shfl(v, src, 64); }

// mask of the lanes of the wave for which `p` holds; every lane of the wave calls it
inline unsigned long long __ballot(bool p)
{
    const int t = (int)threadIdx.x;
    emu::g_exchange[t] = p ? 1 : 0;
    wave_sync();
    unsigned long long m = 0;
    for (int l = 0; l < 64 && (t & ~63) + l < (int)blockDim.x; ++l)
        if (emu::g_exchange[(t & ~63) + l]) m |= 1ull << l;
    wave_sync();
    return m;
}

// value of lane (lane ^ d) of the same wave; every lane of the wave calls it
inline int __shfl_xor(int v, int d, int)
{
    const int t = (int)threadIdx.x;
    emu::g_exchange[t] = v;
    wave_sync();
    const int r = emu::g_exchange[t ^ d];
    wave_sync();
    return r;
}

// global -> LDS copy of `size` bytes per lane: lane l writes to ldsbase + l*size
inline void __builtin_amdgcn_global_load_lds(const void* src, void* ldsbase, int size, int offset, int)
{
    wave_sync();                       // no lane of the wave still reads what is overwritten
    const int lane = (int)threadIdx.x & 63;
    char* dst = (char*)ldsbase + offset + lane * size;
    emu::check_global(src, (size_t)size, "global -> LDS source");
    if (dst < emu::g_lds_lo || dst + size > emu::g_lds_hi) {
        std::fprintf(stderr, "EMU: global -> LDS destination outside the LDS array\n");
        std::abort();
    }
    std::memcpy(dst, src, (size_t)size);
}

namespace emu {
// the same by the lanes for which `active` holds; every lane of the wave calls it
inline void global_load_lds_if(bool active, const void* src, void* ldsbase, int size)
{
    wave_sync();
    if (!active) return;
    const int lane = (int)threadIdx.x & 63;
    char* dst = (char*)ldsbase + lane * size;
    check_global(src, (size_t)size, "global -> LDS source");
    if (dst < g_lds_lo || dst + size > g_lds_hi) {
        std::fprintf(stderr, "EMU: global -> LDS destination outside the LDS array\n");
        std::abort();
    }
    std::memcpy(dst, src, (size_t)size);
}
}  // namespace emu
