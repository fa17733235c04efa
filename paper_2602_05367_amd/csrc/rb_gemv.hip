// Single-op decode kernel: y = sum_k g_k (.) (B_k (h_k (.) x)) for one token of one layer
// (Section 4.1, Eq. (stacked binary weight)) in one launch, nothing prepared beforehand.
//
// The persistent stack kernel needs a plan in the workspace (tables, step lists, the expanded
// input in HBM); for a single call that set-up is several launches and dominates.  Here each
// workgroup (one per compute unit) does the whole of it for itself:
//   a1  the power-of-two scale of each path from max|h_k|, then u_k = h_k (.) x expanded into the
//       four bf8 terms, written into LDS in the register image the MFMA wants (rb_mx.h);
//   a2  its share of row tiles, cut into one run per compute wavefront exactly as the stack
//       kernel cuts it; sign tiles come straight from HBM into registers, a few tiles ahead;
//   a3  the partial sums of the wavefronts meet in LDS;
//   a4  y = sum_k g_k * acc_k, rounded to fp16 once.
// Every rounding step is the stack kernel's (rb_mx_device.h) and sums run in the same order, so
// a layer gives the same bits here and as an op of a stack.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"
#include "rb_internal.h"
#include "rb_layout.h"
#include "rb_mx.h"
#include "rb_mx_device.h"

namespace rb {
namespace gemv1 {

using namespace rb::mx;

constexpr int CW = cwaves_of(1);          // compute wavefronts: the stack kernel's cut of a share
constexpr int WAVES = 16;
constexpr int THREADS = WAVES * 64;
constexpr int DEPTH = 4;                  // sign tiles requested before the first is used
constexpr int MAX_UP_BYTES = 96 * 1024;   // expanded input in LDS: up to 12288 input columns
constexpr int PART_FLOATS = MAXSLOT * CW * 2 * 16;   // [slot][wavefront][path][row]

__global__ __launch_bounds__(THREADS, 1) void gemv1_kernel(const v4u *__restrict__ bits, const __half *__restrict__ g,
                                                           const __half *__restrict__ h, const __half *__restrict__ x,
                                                           __half *__restrict__ y, int out, int in, int RT, int CT)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int n_up = (int)up_bytes(in, 1);
    uint8_t *const up = lds;
    float *const part = reinterpret_cast<float *>(lds + n_up);
    float *const red = part + PART_FLOATS;                       // [path][wavefront]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- scale of each path's input scales (the whole vector, every workgroup for itself)
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        float m = 0.f;
        for (int j = tid; j < in; j += THREADS) m = fmaxf(m, fabsf(__half2float(h[(size_t)p * in + j])));
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
        if (lane == 0) red[p * WAVES + wave] = m;
    }
    // ---- zero: padding columns of the expanded input, partial sums of wavefronts without tiles
    for (int i = tid; i < n_up / 16; i += THREADS) reinterpret_cast<uint4 *>(up)[i] = make_uint4(0, 0, 0, 0);
    for (int i = tid; i < PART_FLOATS; i += THREADS) part[i] = 0.f;
    __syncthreads();
    float sc[2], inv_sc[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        float m = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) m = fmaxf(m, red[p * WAVES + w]);
        sc[p] = input_scale(m);
        inv_sc[p] = 1.f / sc[p];
    }
    // ---- a1: u_k = h_k (.) x as four bf8 terms, in operand order
    for (int j = tid; j < in; j += THREADS) {
        const float xv = __half2float(x[j]);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const uint32_t terms = expand4(__half2float(h[(size_t)p * in + j]) * xv * sc[p]);
#pragma unroll
            for (int t = 0; t < 4; ++t) up[up_offset(1, 0, p, t, j)] = (uint8_t)(terms >> (8 * t));
        }
    }
    __syncthreads();

    // ---- a2, a3: this workgroup's row tiles
    uint32_t rt0, nrt;
    group_rows((uint32_t)RT, blockIdx.x, gridDim.x, 0, rt0, nrt);
    if (wave < CW) {
        const uint32_t uCT = (uint32_t)CT;
        const uint32_t U = nrt * uCT, u0 = (uint32_t)wave * U / CW, u1 = ((uint32_t)wave + 1) * U / CW;
        const int col = lane & 15, qd = lane >> 4, quad = col >> 2;
        const int scale_b = term_scale(col);
        const uint32_t c22 = 0x22222222u;
        // tiles of a share are consecutive in the native layout: tile u of the share is rt0 * CT + u
        const v4u *const tiles = bits + ((size_t)rt0 * uCT) * 64 + lane;
        v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
        for (uint32_t u = u0; u < u1; u += DEPTH) {
            v4u w[DEPTH];
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                w[d] = u + d < u1 ? __builtin_nontemporal_load(tiles + (size_t)(u + d) * 64) : (v4u){0u, 0u, 0u, 0u};
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                if (u + d >= u1) break;
                const uint32_t ct = (u + d) % uCT, slot = (u + d) / uCT;
                const v4i r0 = *reinterpret_cast<const v4i *>(up + (size_t)(ct * 2) * 1024 + lane * 16);
                const v4i r1 = *reinterpret_cast<const v4i *>(up + (size_t)(ct * 2 + 1) * 1024 + lane * 16);
                // lanes 0..7 of a row of 16 hold the first four registers of their operand column,
                // the other four sit eight lanes further on
                v8i b0, b1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    b0[i] = r0[i];
                    b0[4 + i] = __builtin_amdgcn_update_dpp(0, r0[i], 0x108, 0xf, 0xf, true);
                    b1[i] = r1[i];
                    b1[4 + i] = __builtin_amdgcn_update_dpp(0, r1[i], 0x108, 0xf, 0xf, true);
                }
                acc0 = mfma_signs(w[d].x, b0, acc0, c22, scale_b);
                acc1 = mfma_signs(w[d].y, b0, acc1, c22, scale_b);
                acc0 = mfma_signs(w[d].z, b1, acc0, c22, scale_b);
                acc1 = mfma_signs(w[d].w, b1, acc1, c22, scale_b);
                if (ct == uCT - 1 || u + d == u1 - 1) {
                    // the partial sums of this wavefront for the row tile: the first lane of each quad
                    // of operand columns 0..7 holds rows 4 qd .. 4 qd + 3 of path quad
                    v4f v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = quad_sum((quad & 1) ? acc1[r] : acc0[r]);
                    if ((col & 3) == 0 && col < 8)
                        *reinterpret_cast<v4f *>(part + ((slot * CW + wave) * 2 + quad) * 16 + 4 * qd) = v;
                    acc0 = (v4f){0, 0, 0, 0};
                    acc1 = (v4f){0, 0, 0, 0};
                }
            }
        }
    }
    __syncthreads();

    // ---- a4: one thread per row
    if (tid < (int)nrt * 16) {
        const int slot = tid >> 4, row = tid & 15;
        const int grow = (int)(rt0 + slot) * 16 + row;
        if (grow < out) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int w = 0; w < CW; ++w) {
                s0 += part[((slot * CW + w) * 2 + 0) * 16 + row];
                s1 += part[((slot * CW + w) * 2 + 1) * 16 + row];
            }
            const float a0 = __half2float(g[grow]) * inv_sc[0];
            const float a1 = __half2float(g[(size_t)out + grow]) * inv_sc[1];
            reinterpret_cast<_Float16 *>(y)[grow] = (_Float16)path_sum(a0, s0, a1, s1);   // round to nearest even
        }
    }
}

static size_t lds_bytes(const rb_layer *L) { return up_bytes(L->in, 1) + (PART_FLOATS + 2 * WAVES) * sizeof(float); }

bool supported(const rb_layer *L, int T)
{
    const int G = device_groups();
    return T == 1 && L->K == 2 && L->in % 32 == 0 && up_bytes(L->in, 1) <= (size_t)MAX_UP_BYTES && G > 0 &&
           (row_tiles(L->out) + G - 1) / G <= MAXSLOT;
}

int launch(const rb_layer *L, const void *x, void *y, hipStream_t stream)
{
    const int G = device_groups();
    if (G <= 0) return RB_ERR_HIP;
    const size_t lds = lds_bytes(L);
    // once per device: allow the largest LDS request this kernel ever makes
    static bool allowed[64] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return RB_ERR_HIP;
    if (!allowed[dev]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemv1_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                MAX_UP_BYTES + (int)((PART_FLOATS + 2 * WAVES) * sizeof(float))) != hipSuccess)
            return RB_ERR_HIP;
        allowed[dev] = true;
    }
    hipLaunchKernelGGL(gemv1_kernel, dim3(G), dim3(THREADS), lds, stream, static_cast<const v4u *>(L->bits),
                       reinterpret_cast<const __half *>(L->g), reinterpret_cast<const __half *>(L->h),
                       static_cast<const __half *>(x), static_cast<__half *>(y), L->out, L->in, row_tiles(L->out),
                       col_tiles(L->in));
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

}  // namespace gemv1
}  // namespace rb
