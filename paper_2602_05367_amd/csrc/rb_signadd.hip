// Generic residual-binary GEMV: sign-bit XOR + fp32 add.
//
// Section 4.1: y = g (.) (B (h (.) x)) needs only additions and subtractions;
// Eq. (stacked binary weight): the K paths accumulate into one output.
// This kernel is the direct form of that statement and accepts every shape the
// library supports (any out, in % 32 == 0, K = 1, 2 or 3, any T via grid.y).  The
// matrix-core kernels are faster where they apply; this one is the fallback.
//
// One workgroup of eight wavefronts owns one 16-row tile; the wavefronts share out its column
// tiles.  The scaled input u_k = h_k (.) x is staged in LDS in fp32, one column segment at a
// time; each lane applies the 32 signs of each of its words by XOR-ing the bit into the sign of u
// and adding; the four lanes that share a row are summed with two cross-lane shuffles, the eight
// wavefronts through LDS; y = sum_k g_k * acc_k is rounded once.  (A first version gave a
// wavefront a whole row tile: the serial walk over the columns took 3 us per tile and 22-120 us
// per matrix whatever the number of rows.)
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"
#include "rb_layout.h"
#include "rb_device.h"

namespace rb {

constexpr int SIGNADD_SEG_TILES = 16;                          // column tiles staged per pass
constexpr int SIGNADD_SEG_COLS = SIGNADD_SEG_TILES * TILE_COLS;  // 4096 columns
constexpr int SIGNADD_WAVES = 8;

__device__ __forceinline__ float signed_sum32(uint32_t word, const float *__restrict__ u)
{
    // sum over the 32 columns b of (sign bit of column b ? -u[b] : +u[b]); the bit of column b
    // sits at native_bit(b) of the word; u is 16-byte aligned LDS
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
    for (int b = 0; b < 32; b += 4) {
        const float4 v = *reinterpret_cast<const float4 *>(u + b);
        acc0 += __uint_as_float(__float_as_uint(v.x) ^ ((word << (31 - native_bit(b))) & 0x80000000u));
        acc1 += __uint_as_float(__float_as_uint(v.y) ^ ((word << (31 - native_bit(b + 1))) & 0x80000000u));
        acc2 += __uint_as_float(__float_as_uint(v.z) ^ ((word << (31 - native_bit(b + 2))) & 0x80000000u));
        acc3 += __uint_as_float(__float_as_uint(v.w) ^ ((word << (31 - native_bit(b + 3))) & 0x80000000u));
    }
    return (acc0 + acc1) + (acc2 + acc3);
}

template <int K, typename ActT>
__global__ __launch_bounds__(SIGNADD_WAVES * 64) void signadd_gemv_kernel(
    const uint32_t *__restrict__ bits, const __half *__restrict__ g, const __half *__restrict__ h,
    const ActT *__restrict__ X, void *__restrict__ Y, int out_dtype, int out, int in)
{
    __shared__ __attribute__((aligned(16))) float u[K][SIGNADD_SEG_COLS];
    __shared__ float red[SIGNADD_WAVES][K][TILE_ROWS];

    const int t = blockIdx.y;
    const ActT *x = X + (size_t)t * in;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rt = blockIdx.x;
    const int CT = col_tiles(in);
    const int r = lane & 15, q = lane >> 4;

    float acc[K];
#pragma unroll
    for (int k = 0; k < K; ++k) acc[k] = 0.f;

    for (int seg = 0; seg < CT; seg += SIGNADD_SEG_TILES) {
        const int col0 = seg * TILE_COLS;
        __syncthreads();
        for (int j = threadIdx.x; j < SIGNADD_SEG_COLS; j += blockDim.x) {
            const int col = col0 + j;
            const float xv = col < in ? to_float(x[col]) : 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k)
                u[k][j] = col < in ? __half2float(h[(size_t)k * in + col]) * xv : 0.f;
        }
        __syncthreads();
        const int ct_end = min(CT, seg + SIGNADD_SEG_TILES);
        for (int ct = seg + wave; ct < ct_end; ct += SIGNADD_WAVES) {
            const uint32_t *tile = bits + ((size_t)rt * CT + ct) * tile_words(K) + lane * 2 * K;
            uint32_t w[2 * K];
            if constexpr (K == 2) {
                const uint4 v = *reinterpret_cast<const uint4 *>(tile);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            } else if constexpr (K == 3) {
                // 24 bytes per lane, 8-byte aligned: words [c][k] = c * 3 + k
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const uint2 v = reinterpret_cast<const uint2 *>(tile)[i];
                    w[2 * i] = v.x; w[2 * i + 1] = v.y;
                }
            } else {
                const uint2 v = *reinterpret_cast<const uint2 *>(tile);
                w[0] = v.x; w[1] = v.y;
            }
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int j = (ct - seg) * TILE_COLS + 128 * c + 32 * q;
#pragma unroll
                for (int k = 0; k < K; ++k) acc[k] += signed_sum32(w[c * K + k], &u[k][j]);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        acc[k] += __shfl_xor(acc[k], 16);
        acc[k] += __shfl_xor(acc[k], 32);
        if (q == 0) red[wave][k][r] = acc[k];
    }
    __syncthreads();
    const int row = rt * TILE_ROWS + r;
    if (wave == 0 && q == 0 && row < out) {
        float y = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < SIGNADD_WAVES; ++w) a += red[w][k][r];
            y += __half2float(g[(size_t)k * out + row]) * a;
        }
        store_out(Y, out_dtype, (size_t)t * out + row, y);
    }
}

int launch_signadd(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                   hipStream_t stream)
{
    const dim3 grid(row_tiles(L->out), T);
    const dim3 block(SIGNADD_WAVES * 64);
    const uint32_t *bits = static_cast<const uint32_t *>(L->bits);
    const __half *g = reinterpret_cast<const __half *>(L->g);
    const __half *h = reinterpret_cast<const __half *>(L->h);
#define RB_LAUNCH(KK, ACT)                                                                   \
    hipLaunchKernelGGL((signadd_gemv_kernel<KK, ACT>), grid, block, 0, stream, bits, g, h,  \
                       static_cast<const ACT *>(X), Y, out_dtype, L->out, L->in)
    if (act_dtype == RB_F16) {
        if (L->K == 1) RB_LAUNCH(1, __half); else if (L->K == 2) RB_LAUNCH(2, __half); else RB_LAUNCH(3, __half);
    } else {
        if (L->K == 1) RB_LAUNCH(1, bf16_t); else if (L->K == 2) RB_LAUNCH(2, bf16_t); else RB_LAUNCH(3, bf16_t);
    }
#undef RB_LAUNCH
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

}  // namespace rb
