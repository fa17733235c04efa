// Device arithmetic shared by the matrix-core decode kernels (the persistent stack kernel and the
// single-op kernel): both must produce the same bits for the same op, so everything that rounds
// lives here once.  See rb_mx.h for the formats.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <cstdint>

#include "rb_mx.h"

namespace rb {
namespace mx {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// power-of-two scale of one path's input scales: max|h| * sc lies in [1/4, 1/2), so that
// |h x sc| < 2^15 for any fp16 x (1 for an all-zero or non-finite h)
__device__ __forceinline__ float input_scale(float max_abs_h)
{
    float sc = 1.f;
    if (max_abs_h > 0.f && max_abs_h < INFINITY) {
        int e;
        frexpf(max_abs_h, &e);              // max_abs_h = f * 2^e, f in [0.5, 1)
        sc = ldexpf(1.f, -e - 1);
    }
    return sc;
}

// four bf8 terms of u: u ~= t0 + t1/8 + t2/64 + t3/512 (each term rounds the rest)
__device__ __forceinline__ uint32_t expand4(float u)
{
    uint32_t out = 0;
    float r = u;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int pk = __builtin_amdgcn_cvt_pk_bf8_f32(r, 0.f, 0, false);
        out |= (uint32_t)(pk & 0xff) << (8 * t);
        // (r - term) * 8: the difference is exact (|u| < 2^15 never saturates a term), so one fused
        // multiply-add on 8 r, which does not wait for the conversions, gives the same bits
        r = __builtin_fmaf(-__builtin_amdgcn_cvt_f32_bf8(pk, 0), 8.f, r * 8.f);
    }
    // A value that is not finite (an fp16 overflow upstream) becomes four NaN terms of one fixed
    // pattern, so that the product is NaN whatever the conversion would have made of it and no
    // term byte is ever 0xff, which the stack kernel reads as "not written yet".
    return fabsf(u) < __builtin_inff() ? out : 0x7e7e7e7eu;
}

// byte address of (token, path, term, input column j) in an op's expanded input
__device__ __forceinline__ size_t up_offset(int T, int tok, int p, int t, int j)
{
    return up_group_offset(T, j & ~15, 8 * tok + 4 * p + t) + (size_t)(j & 15);
}

// row tiles of an op that workgroup grp (of G) owns: [rt0, rt0 + nrt).  Shares differ by one row
// tile when G does not divide RT, and the larger ones sit at the same places for every op of that
// height (every fourth share for 5120 rows on 256 workgroups); the op at position pos of its stage
// deals its shares starting pos workgroups further on, so that the larger shares of like-shaped ops
// of a stage fall on different workgroups where they can.
__host__ __device__ inline void group_rows(uint32_t RT, uint32_t grp, uint32_t G, int pos, uint32_t &rt0, uint32_t &nrt)
{
    if ((G & (G - 1)) == 0) {                 // the usual number of workgroups is a power of two
        const int shift = __builtin_ctz(G);
        const uint32_t g = (grp + (uint32_t)pos) & (G - 1);
        rt0 = (g * RT) >> shift;
        nrt = (((g + 1) * RT) >> shift) - rt0;
        return;
    }
    const uint32_t g = (grp + (uint32_t)pos) % G;
    rt0 = g * RT / G;
    nrt = (g + 1) * RT / G - rt0;
}

// 16 rows x 128 columns of one path's signs (one word per lane, see rb_layout.h) times the 16
// operand columns of b, accumulated into acc
__device__ __forceinline__ v4f mfma_signs(uint32_t w, v8i b, v4f acc, uint32_t c22, int scale_b)
{
    v8i a;
    a[0] = (int)(((w << 3) & 0x88888888u) | c22);
    a[1] = (int)(((w << 2) & 0x88888888u) | c22);
    a[2] = (int)(((w << 1) & 0x88888888u) | c22);
    a[3] = (int)((w & 0x88888888u) | c22);
    a[4] = 0; a[5] = 0; a[6] = 0; a[7] = 0;
    // A: fp4 (cbsz = 4), B: bf8 (blgp = 1); scale bytes are E8M0 exponents
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 1, 0, 0x7f7f7f7f, 0, scale_b);
}

// E8M0 scale bytes of the right operand for the lane that holds operand column col: term t = col % 4
// carries the factor 8^-t
__device__ __forceinline__ int term_scale(int col) { return (127 - 3 * (col & 3)) * 0x01010101; }

// the value of lane ^ 16: the 16-lane rows swapped in registers, no trip through LDS
// (v_permlane16_swap_b32 with both operands v: its first result holds, in the odd rows, what the
// even row before them had; its second result, in the even rows, what the odd row after them had).
// A lane and its partner must both be active.
__device__ __forceinline__ float xor16(float v)
{
    const unsigned x = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    return __uint_as_float((threadIdx.x & 16u) ? r[0] : r[1]);
}
// the same for lane ^ 32: the halves of the wavefront swapped (v_permlane32_swap_b32)
__device__ __forceinline__ float xor32(float v)
{
    const unsigned x = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return __uint_as_float((threadIdx.x & 32u) ? r[0] : r[1]);
}
// sum over the 16 lanes of a row, left in all of them: two exchanges inside the quad, then the
// mirrored lane of the eight (in the other quad, whose four lanes hold the same sum) and of the row
__device__ __forceinline__ float row_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    return v;
}

// The 16 lanes of a row hold one word of four bytes each (lane r: bytes b_r0 .. b_r3); afterwards
// lane t < 4 of the row holds the 16 bytes b_0t .. b_15t.  Two exchanges inside each quad with a
// byte select each (a 4 x 4 byte transpose over four lanes), then three row shifts bring the
// quads' words together.  The whole row must be active.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_move(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ v4i transpose_16x4_bytes(uint32_t w)
{
    const uint32_t lane = threadIdx.x;
    const uint32_t x = dpp_move<0xB1>(w);                                           // quad_perm [1,0,3,2]
    const uint32_t a = __builtin_amdgcn_perm(x, w, (lane & 1) ? 0x03070105u : 0x06020400u);
    const uint32_t y = dpp_move<0x4E>(a);                                           // quad_perm [2,3,0,1]
    const uint32_t z = __builtin_amdgcn_perm(y, a, (lane & 2) ? 0x03020706u : 0x05040100u);
    v4i v;
    v[0] = (int)z;
    v[1] = (int)dpp_move<0x104>(z);                                                 // row_shl:4: the lane four further on
    v[2] = (int)dpp_move<0x108>(z);
    v[3] = (int)dpp_move<0x10C>(z);
    return v;
}

// sum over the four lanes of a quad (the four terms of one path and token)
__device__ __forceinline__ float quad_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));   // 1,0,3,2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));   // 2,3,0,1
    return v;
}

// y = (g_1 / sc_1) * acc_1 + (g_2 / sc_2) * acc_2, one rounding of the product of path 2 and one of the sum
__device__ __forceinline__ float path_sum(float a0, float s0, float a1, float s1)
{
    return __builtin_fmaf(a0, s0, a1 * s1);
}

}  // namespace mx
}  // namespace rb
