// Comparators reported next to the binary path: a dense fp16 GEMV (the
// full-precision row of the paper's inference table, written for this GPU) and
// a pure streaming read (the read-bandwidth ceiling of the device).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"

namespace rb {

constexpr int DENSE_WAVES = 4;      // wavefronts per workgroup
constexpr int DENSE_ROWS = 4;       // rows per wavefront

// One wavefront computes DENSE_ROWS dot products; every lane walks the row in
// 16-byte (8 x fp16) steps, 512 columns per wavefront step.
__global__ __launch_bounds__(DENSE_WAVES * 64) void dense_gemv_f16_kernel(
    const __half *__restrict__ W, const __half *__restrict__ x, __half *__restrict__ y, int out, int in)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * DENSE_WAVES + wave) * DENSE_ROWS;
    if (row0 >= out) return;
    float acc[DENSE_ROWS];
#pragma unroll
    for (int r = 0; r < DENSE_ROWS; ++r) acc[r] = 0.f;
    for (int j = lane * 8; j < in; j += 64 * 8) {
        const uint4 xv = *reinterpret_cast<const uint4 *>(x + j);
        const __half2 *xh = reinterpret_cast<const __half2 *>(&xv);
#pragma unroll
        for (int r = 0; r < DENSE_ROWS; ++r) {
            const int row = min(row0 + r, out - 1);
            const uint4 wv = *reinterpret_cast<const uint4 *>(W + (size_t)row * in + j);
            const __half2 *wh = reinterpret_cast<const __half2 *>(&wv);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 a = __half22float2(wh[e]), b = __half22float2(xh[e]);
                acc[r] = fmaf(a.x, b.x, acc[r]);
                acc[r] = fmaf(a.y, b.y, acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < DENSE_ROWS; ++r) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) acc[r] += __shfl_xor(acc[r], off);
        if (lane == 0 && row0 + r < out) y[row0 + r] = __float2half_rn(acc[r]);
    }
}

constexpr int STREAM_GROUPS = 256 * 8;
constexpr int STREAM_THREADS = 256;

__global__ __launch_bounds__(STREAM_THREADS) void stream_read_kernel(
    const uint4 *__restrict__ src, size_t n16, uint4 *__restrict__ sink)
{
    uint4 acc = make_uint4(0, 0, 0, 0);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    // four independent loads in flight per lane
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z; acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        acc.x ^= __shfl_xor(acc.x, off); acc.y ^= __shfl_xor(acc.y, off);
        acc.z ^= __shfl_xor(acc.z, off); acc.w ^= __shfl_xor(acc.w, off);
    }
    __shared__ uint4 part[STREAM_THREADS / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint4 s = part[0];
        for (int w = 1; w < STREAM_THREADS / 64; ++w) {
            s.x ^= part[w].x; s.y ^= part[w].y; s.z ^= part[w].z; s.w ^= part[w].w;
        }
        sink[blockIdx.x] = s;
    }
}

}  // namespace rb

extern "C" int rb_dense_gemv_f16(const uint16_t *W, const uint16_t *x, uint16_t *y, int out, int in,
                                 void *stream)
{
    if (!W || !x || !y) return RB_ERR_NULL;
    if (out < 1 || in < 8 || in % 8 != 0) return RB_ERR_SHAPE;
    if (((uintptr_t)W | (uintptr_t)x) & 15) return RB_ERR_ALIGN;
    const int rows_per_group = rb::DENSE_WAVES * rb::DENSE_ROWS;
    hipLaunchKernelGGL(rb::dense_gemv_f16_kernel, dim3((out + rows_per_group - 1) / rows_per_group),
                       dim3(rb::DENSE_WAVES * 64), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const __half *>(W), reinterpret_cast<const __half *>(x),
                       reinterpret_cast<__half *>(y), out, in);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

extern "C" int rb_stream_read_groups(void) { return rb::STREAM_GROUPS; }

extern "C" int rb_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return RB_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return RB_ERR_SHAPE;
    if (((uintptr_t)src | (uintptr_t)sink) & 15) return RB_ERR_ALIGN;
    hipLaunchKernelGGL(rb::stream_read_kernel, dim3(rb::STREAM_GROUPS), dim3(rb::STREAM_THREADS), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(src), bytes / 16,
                       static_cast<uint4 *>(sink));
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}
