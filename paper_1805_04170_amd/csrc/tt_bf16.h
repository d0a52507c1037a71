// fp32 -> bf16 conversions used by every kernel that stores bf16 (round to nearest even).
#pragma once
#include "tt_device.h"
#include <cstdint>

namespace tt {

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u; // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                  // round to nearest even
}

// two floats -> packed bf16 pair (low half = a); round to nearest even, compiled to v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v = {(__bf16)a, (__bf16)b};
    return *reinterpret_cast<uint32_t *>(&v);
}

} // namespace tt
