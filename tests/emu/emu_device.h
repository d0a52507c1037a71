// Host stand-ins for what the tile engines take from the device tool chain (see csrc/tt_device.h).  One thread of one
// workgroup runs at a time; barriers, wait counts and scheduling hints do nothing (no thread's addresses depend on
// another thread's data); MFMAs return their accumulator; every global and LDS access is a real host access into
// buffers of exactly the size the launch was given, checked here and by the address sanitizer.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#define __device__
#define __host__
#define __global__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))

struct EmuDim3 { unsigned x, y, z; };
inline EmuDim3 threadIdx, blockIdx;

inline uint32_t __float_as_uint(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float __uint_as_float(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
inline int __popc(uint32_t v) { return __builtin_popcount(v); }

#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_iglp_opt(x) ((void)0)
#ifdef TT_EMU_LOCKSTEP
#include "emu_lockstep.h"
#else
inline void __syncthreads() {}
#define __builtin_amdgcn_s_waitcnt(x) ((void)0)
#define __builtin_amdgcn_wave_barrier() ((void)0)
#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) (c)
#endif

// ---- the little of the HIP host API that the launch code of a .hip file uses: a launch runs the kernel for every thread
// of every workgroup in turn (no thread of the emulated kernels reads what another thread wrote)
struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
typedef void *hipStream_t;
enum hipError_t { hipSuccess = 0 };
enum hipFuncAttribute { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void *, hipFuncAttribute, int) { return hipSuccess; }
// streams and events: everything here runs at once and in order
typedef void *hipEvent_t;
enum { hipEventDisableTiming = 2 };
inline hipError_t hipEventCreate(hipEvent_t *e) { *e = reinterpret_cast<hipEvent_t>(1); return hipSuccess; }
inline hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = reinterpret_cast<hipEvent_t>(1); return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
// a `__device__` array is a plain host array here, and its "device address" is its own
#define HIP_SYMBOL(x) (x)
inline hipError_t hipGetSymbolAddress(void **p, const void *symbol) { *p = const_cast<void *>(symbol); return hipSuccess; }
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 63 };
inline hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
inline hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t, int)
{
    // MI355X: 256 CUs (EMU_CUS: a smaller device, so that small products give a persistent workgroup several tiles)
    const char *e = std::getenv("EMU_CUS");
    *value = e ? std::atoi(e) : 256;
    return hipSuccess;
}
// LDS arrays: one copy for the whole process (one workgroup runs at a time), whether a kernel declares them inside its
// body or as `extern __shared__ T name[]`, which the driver then defines with the same storage class
#define __shared__ thread_local
inline unsigned long long g_emu_threads_run = 0;
// kernels that declare `extern __shared__ T name[]`: whoever defines the array registers it here; a launch then makes
// everything past its dynamic size inaccessible to the address sanitizer (several arrays: one name per kernel family)
struct EmuLds { char *base; size_t cap; };
inline EmuLds g_emu_lds[8];
inline int g_emu_lds_n = 0;
inline int emu_register_lds(void *base, size_t cap)
{
    if (g_emu_lds_n == 8) { std::fprintf(stderr, "EMU: too many LDS arrays\n"); std::abort(); }
    g_emu_lds[g_emu_lds_n++] = {static_cast<char *>(base), cap};
    return g_emu_lds_n;
}
#ifdef TT_EMU_LOCKSTEP // built without the address sanitizer (it does not follow fibers): the explicit range checks remain
inline void __asan_poison_memory_region(void const volatile *, size_t) {}
inline void __asan_unpoison_memory_region(void const volatile *, size_t) {}
#else
extern "C" void __asan_poison_memory_region(void const volatile *addr, size_t size);
extern "C" void __asan_unpoison_memory_region(void const volatile *addr, size_t size);
#endif
void emu_set_lds_limit(size_t dyn_bytes); // defined below, after tt::dev
template <class F> inline void emu_launch(F &&body, dim3 grid, dim3 block, size_t dyn_bytes)
{
    for (int i = 0; i < g_emu_lds_n; ++i) {
        if (dyn_bytes > g_emu_lds[i].cap) { std::fprintf(stderr, "EMU FAULT: launch asks for %zu bytes of LDS\n", dyn_bytes); std::abort(); }
        __asan_unpoison_memory_region(g_emu_lds[i].base, g_emu_lds[i].cap);
        __asan_poison_memory_region(g_emu_lds[i].base + dyn_bytes, g_emu_lds[i].cap - dyn_bytes);
    }
    emu_set_lds_limit(dyn_bytes);
    for (unsigned by = 0; by < grid.y; ++by)
        for (unsigned b = 0; b < grid.x; ++b) {
            blockIdx = {b, by, 0};
#ifdef TT_EMU_LOCKSTEP
            emu::run_block(body, block.x);
            g_emu_threads_run += block.x;
#else
            for (unsigned t = 0; t < block.x; ++t) {
                threadIdx = {t, 0, 0};
                body();
                ++g_emu_threads_run;
            }
#endif
        }
}
#define hipLaunchKernelGGL(kern, grid, block, smem, stream, ...) emu_launch([&]() { kern(__VA_ARGS__); }, grid, block, smem)

namespace tt {
namespace dev {

typedef short s16x4 __attribute__((ext_vector_type(4)));

struct Region { const char *lo, *hi; };
inline char *g_lds = nullptr;    // the workgroup's LDS
inline size_t g_lds_bytes = 0;
inline Region g_readable[192];   // operand buffers of the launch (none registered: reads are not range-checked here)
inline int g_n_readable = 0;
inline unsigned long long g_dma_bytes = 0;

[[noreturn]] inline void fail(const char *what, const void *addr, size_t n)
{
    std::fprintf(stderr, "EMU FAULT: %s at %p (+%zu) block %u thread %u\n", what, addr, n, blockIdx.x, threadIdx.x);
    std::abort();
}

inline uint32_t lds_addr(char *p)
{
    // with several named LDS arrays in the build: the one the pointer lies in is this kernel's LDS
    for (int i = 0; i < g_emu_lds_n; ++i)
        if (p >= g_emu_lds[i].base && p <= g_emu_lds[i].base + g_emu_lds[i].cap) g_lds = g_emu_lds[i].base;
    if (p < g_lds || p > g_lds + g_lds_bytes) fail("pointer outside LDS", p, 0);
    return (uint32_t)(p - g_lds);
}

inline void check_read(const char *g, size_t n)
{
    if (g_n_readable == 0) return;
    for (int i = 0; i < g_n_readable; ++i)
        if (g >= g_readable[i].lo && g + n <= g_readable[i].hi) return;
    fail("global read outside every operand", g, n);
}

inline void land16(const char *g, uint32_t lds_wave_addr)
{
    const uint32_t dst = lds_wave_addr + (threadIdx.x & 63u) * 16u;
    if ((size_t)dst + 16 > g_lds_bytes) fail("load lands outside LDS", g_lds + dst, 16);
    if ((uintptr_t)g % 16) fail("misaligned 16-byte global -> LDS load", g, 16);
    check_read(g, 16);
#ifdef TT_EMU_LOCKSTEP
    emu::issue_lds_load(g_lds + dst, g);
#else
    std::memcpy(g_lds + dst, g, 16);
#endif
    g_dma_bytes += 16;
}

inline void lds_dma16(const void *g, uint32_t lds_wave_addr) { land16(static_cast<const char *>(g), lds_wave_addr); }
inline void lds_dma16(uint32_t lane_offset, uint64_t uniform_base, uint32_t lds_wave_addr)
{
    land16(reinterpret_cast<const char *>(uniform_base) + lane_offset, lds_wave_addr);
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool NON_TEMPORAL> inline void store16(void *p, u32x4_t v)
{
    if ((uintptr_t)p % 16) fail("misaligned 16-byte global store", p, 16);
    std::memcpy(p, &v, 16);
#ifdef TT_EMU_LOCKSTEP
    emu::issue_counted_store();
#endif
}

inline s16x4 lds_read_tr16_b64(const char *a)
{
    if (a < g_lds || a + 8 > g_lds + g_lds_bytes) fail("LDS transpose read outside LDS", a, 8);
    s16x4 v;
#ifdef TT_EMU_LOCKSTEP
    std::memcpy(emu::my_wave().tr[emu::lane()], a, 8);
    emu::transpose_groups_of_16();
    std::memcpy(&v, emu::my_wave().tr[emu::lane()], 8);
#else
    std::memcpy(&v, a, 8);
#endif
    return v;
}

} // namespace dev
} // namespace tt

inline void emu_set_lds_limit(size_t dyn_bytes)
{
    if (g_emu_lds_n > 0) tt::dev::g_lds_bytes = dyn_bytes;
}

