// Small device helpers shared by the kernels of this library: element types,
// conversions and the fp32 -> output store.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <cstdint>

#include "rabit.h"

namespace rb {

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

// fp32 -> bfloat16, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void store_out(void *Y, int out_dtype, size_t idx, float v)
{
    if (out_dtype == RB_F16) {
        static_cast<__half *>(Y)[idx] = __float2half_rn(v);
    } else if (out_dtype == RB_BF16) {
        static_cast<uint16_t *>(Y)[idx] = f32_to_bf16_rne(v);
    } else {
        static_cast<float *>(Y)[idx] = v;
    }
}

// OR over each group of eight consecutive lanes, left in all eight: two exchanges inside the quad,
// then one with the mirrored lane of the group (7 - i, which sits in the other quad).  Data-parallel
// moves: every lane of the wavefront must be active.
__device__ __forceinline__ uint32_t or_over_8(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);   // row_half_mirror
    return v;
}

}  // namespace rb
