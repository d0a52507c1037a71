// The few things the tile engines need from the device tool chain that have no meaning on a CPU, in one place:
// the address of a shared-memory pointer inside LDS, the global -> LDS loads written in assembly, the LDS transpose
// read.  The device build gets the HIP runtime header and these inline functions.  A host build for checking memory
// accesses (TT_HOST_EMULATION: one thread of one workgroup at a time on the CPU, every global and LDS access a real,
// bounds-checked host access; see tests/emu/) gets stand-ins with the same names from its own emu_device.h.
#pragma once
#ifdef TT_HOST_EMULATION
#include "emu_device.h"
#else
#include <hip/hip_runtime.h>
#include <cstdint>

namespace tt {
namespace dev {

typedef short s16x4 __attribute__((ext_vector_type(4)));

// byte address inside the workgroup's LDS of a pointer into its shared memory
__device__ __forceinline__ uint32_t lds_addr(char *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)p;
}

// global -> LDS, 16 bytes per lane: lane i's chunk lands at lds_wave_addr + 16 i (M0 holds the wave-uniform LDS
// address; s_nop: one wait state between the write of M0 and its use).  Assembly on purpose: for the builtin form the
// compiler's wait-count pass assumes that any later LDS read may alias the incoming data and puts s_waitcnt vmcnt(0) in
// front of the next fragment read; here the waits are the explicit s_waitcnt + barrier pairs of the main loops.
// ... every lane supplies a full global address
__device__ __forceinline__ void lds_dma16(const void *g, uint32_t lds_wave_addr)
{
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "{m0}"(lds_wave_addr), "v"(g) : "memory");
}
// ... a wave-uniform base (scalar registers) plus a 32-bit offset per lane
__device__ __forceinline__ void lds_dma16(uint32_t lane_offset, uint64_t uniform_base, uint32_t lds_wave_addr)
{
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_offset), "s"(uniform_base), "{m0}"(lds_wave_addr) : "memory");
}

// 16-byte global store.  A named function because kernels that leave stores in flight over a wait count them
// (s_waitcnt vmcnt(n) counts a wave's loads and stores alike, in issue order), and the host emulation counts them here.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool NON_TEMPORAL> __device__ __forceinline__ void store16(void *p, u32x4_t v)
{
    if constexpr (NON_TEMPORAL) __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(p));
    else *reinterpret_cast<u32x4_t *>(p) = v;
}

// LDS transpose read: 8 bytes per lane at a, handed out transposed over each group of 16 lanes (four bf16 per lane)
__device__ __forceinline__ s16x4 lds_read_tr16_b64(const char *a)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a);
}

} // namespace dev
} // namespace tt
#endif
