// Training-side kernels of the residual-binary layer (Section 4.2, Alg. 2).
//
//   * rb_couple: the on-the-fly residual coupling of the forward pass.  From the shared
//     full-precision weight and the scales it derives the binary cores path after path,
//     B_i = sign(R_{i-1}), R_i = R_{i-1} - g_i (.) B_i (.) h_i, and writes them packed (canonical
//     words and/or the kernel-native tiles the inference kernels read), so that a training step
//     can run its forward pass through the same kernels as inference.
//   * rb_weight_grad: the effective-weight gradient G = (dL/dY) X^T (Eq. RaBiT-grad-wfp), the
//     straight-through gradient of the shared weight.
//   * rb_scale_grads: the gradients of the scales (Eq. RaBiT-grad-gh) with the binary cores held
//     constant.  Summed over the samples they are signed reductions of G:
//         grad g_i[r] = sum_c B_i[r][c] h_i[c] G[r][c]       (rows)
//         grad h_i[c] = sum_r B_i[r][c] g_i[r] G[r][c]       (columns: the transposed product)
//     so one pass over G per direction gives them for every path, whatever the batch size.
//
// All three are bound by HBM (4 bytes per weight read); none needs matrix cores.  Every sum runs in
// a fixed order, so results do not depend on scheduling.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"
#include "rb_device.h"
#include "rb_internal.h"
#include "rb_layout.h"

namespace rb {
namespace train {

constexpr int ROW_SLICE = 64;          // rows one workgroup of the column reduction walks
constexpr int COUPLE_CHUNK = 1024;     // columns one wavefront of the coupling kernel walks

// ------------------------------------------------------------------ couple ---
__global__ __launch_bounds__(256) void zero_kernel(uint32_t *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// One wavefront per row and chunk of COUPLE_CHUNK columns.  A lane takes four consecutive columns
// at a time (one 16-byte load of W; the chunk's loads are all requested before the first is used),
// so a step of the wavefront covers 256 columns and eight lanes hold one sign word between them:
// lane i of the eight has columns 4 i .. 4 i + 3 of the word, bits 4 i + j of the canonical word
// (bit b = column 32 w + b, 1 means -1) and bits 16 (i % 2) + 4 j + i / 2 of the native one (native
// bit 4 e + s is column 8 s + e); each lane shifts its four bits into place in both and an OR over
// the eight lanes gives the words.  The residual is fp32 with one rounding for g * h and one for
// the subtraction, the arithmetic the definition fixes (the sign of the product is exact).
__global__ __launch_bounds__(256) void couple_kernel(const float *__restrict__ W, const __half *__restrict__ g,
                                                     const __half *__restrict__ h, int K, int out, int in,
                                                     uint32_t *__restrict__ packed, uint32_t *__restrict__ native,
                                                     float *__restrict__ residual)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= out) return;
    const int W32 = in / 32, CT = col_tiles(in);
    float gr[RB_MAX_K];
    for (int k = 0; k < K; ++k) gr[k] = __half2float(g[(size_t)k * out + row]);
    const int chunk0 = blockIdx.y * COUPLE_CHUNK;
    constexpr int STEPS = COUPLE_CHUNK / 256;
    float4 wv[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        const int c = chunk0 + 256 * i + 4 * lane;
        wv[i] = c < in ? *reinterpret_cast<const float4 *>(W + (size_t)row * in + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        const int c0 = chunk0 + 256 * i;
        if (c0 >= in) break;
        const int c = c0 + 4 * lane;
        const bool real = c < in;                              // in % 32 == 0: all four columns or none
        float r[4] = {wv[i].x, wv[i].y, wv[i].z, wv[i].w};
        const int i8 = lane & 7;
        const int w = (c0 >> 5) + (lane >> 3);                 // the word this group of eight lanes holds
        for (int k = 0; k < K; ++k) {
            float hv[4] = {0.f, 0.f, 0.f, 0.f};
            if (real) {
                const uint2 hb = *reinterpret_cast<const uint2 *>(h + (size_t)k * in + c);
                hv[0] = __half2float(__ushort_as_half((unsigned short)(hb.x & 0xffffu)));
                hv[1] = __half2float(__ushort_as_half((unsigned short)(hb.x >> 16)));
                hv[2] = __half2float(__ushort_as_half((unsigned short)(hb.y & 0xffffu)));
                hv[3] = __half2float(__ushort_as_half((unsigned short)(hb.y >> 16)));
            }
            uint32_t can = 0, nat = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool neg = real && !(r[j] >= 0.f);       // sign(0) = +1; columns past the end read as +1
                const float prod = __fmul_rn(gr[k], hv[j]);
                r[j] = neg ? __fadd_rn(r[j], prod) : __fsub_rn(r[j], prod);
                can |= neg ? 1u << j : 0u;
                nat |= neg ? 1u << (4 * j) : 0u;
            }
            const uint32_t word = or_over_8(can << (4 * i8));
            const uint32_t nword = or_over_8(nat << (16 * (i8 & 1) + (i8 >> 1)));
            if (i8 == 0 && w < W32) {
                if (packed) packed[((size_t)k * out + row) * W32 + w] = word;
                if (native) {
                    const int rt = row / TILE_ROWS, ct = w / 8, cc = (w % 8) / 4, q = w % 4;
                    native[((size_t)rt * CT + ct) * tile_words(K) + lane_word((row % TILE_ROWS) + 16 * q, cc, k, K)] = nword;
                }
            }
        }
        if (residual && real) *reinterpret_cast<float4 *>(residual + (size_t)row * in + c) = make_float4(r[0], r[1], r[2], r[3]);
    }
}

// --------------------------------------------------------------- gradients ---
// G[r][c] = sum_n Delta[n][r] X[n][c]: one thread per element, the sum over samples in order.
__global__ __launch_bounds__(256) void weight_grad_kernel(const __half *__restrict__ Delta, const __half *__restrict__ X,
                                                          int N, int out, int in, float *__restrict__ G)
{
    const int c = blockIdx.x * 256 + threadIdx.x, r = blockIdx.y;
    if (c >= in) return;
    float s = 0.f;
    for (int n = 0; n < N; ++n) s = __builtin_fmaf(__half2float(Delta[(size_t)n * out + r]), __half2float(X[(size_t)n * in + c]), s);
    G[(size_t)r * in + c] = s;
}

// Both scale gradients from one pass over G.  A wavefront takes a slab of ROW_SLICE rows by 256
// columns, a lane four consecutive columns (one 16-byte load of G and four bits of a sign word per
// row and path), eight rows in flight.  The column sums of grad h stay in the lane (rows in order);
// the row sums of grad g need the whole wavefront: the eight rows of a group are summed together,
// three exchanges that each halve the number of rows a lane carries (after them lane l holds row
// 4 (l & 1) + 2 (l >> 1 & 1) + (l >> 2 & 1) of the group, summed over its eight lanes) and three
// more over the eight-lane groups.  Partial sums: [slice][K][in] and [column block][K][out]; the
// second kernel adds them in order, so results repeat bit for bit.
__global__ __launch_bounds__(64) void grad_slab_kernel(const float *__restrict__ G, const uint32_t *__restrict__ packed,
                                                       const __half *__restrict__ g, const __half *__restrict__ h, int K,
                                                       int out, int in, float *__restrict__ part_h,
                                                       float *__restrict__ part_g)
{
    const int lane = threadIdx.x;
    const int c = (blockIdx.x * 64 + lane) * 4, slice = blockIdx.y;
    const bool real = c < in;                                  // in % 32 == 0: all four columns or none
    const int cs = real ? c : 0;
    const int W32 = in / 32, r0 = slice * ROW_SLICE, r1 = min(out, r0 + ROW_SLICE);
    float sh[RB_MAX_K][4], hv[RB_MAX_K][4];
    for (int k = 0; k < RB_MAX_K; ++k)
        for (int e = 0; e < 4; ++e) {
            sh[k][e] = 0.f;
            hv[k][e] = k < K && real ? __half2float(h[(size_t)k * in + c + e]) : 0.f;
        }
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    const int my_row = 4 * (int)b0 + 2 * (int)b1 + (int)b2;
    for (int rb = r0; rb < r1; rb += 8) {
        float4 gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            gv[u] = real && rb + u < r1 ? *reinterpret_cast<const float4 *>(G + (size_t)(rb + u) * in + c)
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < K; ++k) {
            float rp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = min(rb + u, r1 - 1);             // rows past the end: G read as zero above
                const float v[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                const uint32_t bits4 = packed[((size_t)k * out + r) * W32 + (cs >> 5)] >> (cs & 31);
                const float gk = __half2float(g[(size_t)k * out + r]);
                float rs = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float sv = (bits4 >> e) & 1u ? -v[e] : v[e];
                    sh[k][e] = __builtin_fmaf(gk, sv, sh[k][e]);
                    rs = __builtin_fmaf(hv[k][e], sv, rs);
                }
                rp[u] = rs;
            }
            float q[4], p2[2];
#pragma unroll
            for (int u = 0; u < 4; ++u) q[u] = (b0 ? rp[u + 4] : rp[u]) + __shfl_xor(b0 ? rp[u] : rp[u + 4], 1);
#pragma unroll
            for (int u = 0; u < 2; ++u) p2[u] = (b1 ? q[u + 2] : q[u]) + __shfl_xor(b1 ? q[u] : q[u + 2], 2);
            float o = (b2 ? p2[1] : p2[0]) + __shfl_xor(b2 ? p2[0] : p2[1], 4);
            o += __shfl_xor(o, 8);
            o += __shfl_xor(o, 16);
            o += __shfl_xor(o, 32);
            if (lane < 8 && rb + my_row < r1) part_g[((size_t)blockIdx.x * K + k) * out + rb + my_row] = o;
        }
    }
    if (real)
        for (int k = 0; k < K; ++k)
            *reinterpret_cast<float4 *>(part_h + ((size_t)slice * K + k) * in + c) =
                make_float4(sh[k][0], sh[k][1], sh[k][2], sh[k][3]);
}

// element i < K * in of grad h: the slices in order; the rest, grad g: the column blocks in order
__global__ __launch_bounds__(256) void grad_finish_kernel(const float *__restrict__ part_h, int slices,
                                                          const float *__restrict__ part_g, int col_blocks, int K,
                                                          int out, int in, float *__restrict__ grad_g,
                                                          float *__restrict__ grad_h)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < K * in) {
        float s = 0.f;
#pragma unroll 8
        for (int sl = 0; sl < slices; ++sl) s += part_h[(size_t)sl * K * in + i];
        grad_h[i] = s;
    } else if (i < K * in + K * out) {
        const int j = i - K * in;
        float s = 0.f;
#pragma unroll 8
        for (int cb = 0; cb < col_blocks; ++cb) s += part_g[(size_t)cb * K * out + j];
        grad_g[j] = s;
    }
}

static int check_shape(int K, int out, int in)
{
    return (K < 1 || K > RB_MAX_K || out < 1 || in < 32 || in % 32 != 0) ? RB_ERR_SHAPE : RB_OK;
}

}  // namespace train
}  // namespace rb

using namespace rb::train;

extern "C" int rb_couple(const float *W, const uint16_t *g, const uint16_t *h, int K, int out, int in,
                         uint32_t *packed, void *native, float *residual, void *stream_)
{
    if (!W || !g || !h) return RB_ERR_NULL;
    if (!packed && !native) return RB_ERR_NULL;
    const int rc = check_shape(K, out, in);
    if (rc != RB_OK) return rc;
    if (((uintptr_t)packed | (uintptr_t)native) & 3) return RB_ERR_ALIGN;
    if (((uintptr_t)W | (uintptr_t)residual) & 15) return RB_ERR_ALIGN;
    if ((uintptr_t)h & 7) return RB_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (native) {
        // rows and columns of padding read as +1 (bit 0); a kernel, not a memset, so that a caller may capture the call
        const size_t words = rb_native_bytes(K, out, in) / 4;
        hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                           static_cast<uint32_t *>(native), words);
    }
    hipLaunchKernelGGL(couple_kernel, dim3((unsigned)((out + 3) / 4), (unsigned)((in + COUPLE_CHUNK - 1) / COUPLE_CHUNK)),
                       dim3(256), 0, stream, W,
                       reinterpret_cast<const __half *>(g), reinterpret_cast<const __half *>(h), K, out, in, packed,
                       static_cast<uint32_t *>(native), residual);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

extern "C" int rb_weight_grad(const uint16_t *Delta, const uint16_t *X, int N, int out, int in, float *G, void *stream_)
{
    if (!Delta || !X || !G) return RB_ERR_NULL;
    if (N < 1 || out < 1 || in < 1 || out > 65535) return RB_ERR_SHAPE;
    hipLaunchKernelGGL(weight_grad_kernel, dim3((unsigned)((in + 255) / 256), (unsigned)out), dim3(256), 0,
                       static_cast<hipStream_t>(stream_), reinterpret_cast<const __half *>(Delta),
                       reinterpret_cast<const __half *>(X), N, out, in, G);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

extern "C" size_t rb_scale_grads_workspace_bytes(int K, int out, int in)
{
    if (check_shape(K, out, in) != RB_OK) return 0;
    // [slice][K][in] partial sums of grad h, then [column block][K][out] partial sums of grad g
    return ((size_t)((out + ROW_SLICE - 1) / ROW_SLICE) * K * in + (size_t)((in + 255) / 256) * K * out) * sizeof(float);
}

extern "C" int rb_scale_grads(const float *G, const uint32_t *packed, const uint16_t *g, const uint16_t *h, int K,
                              int out, int in, float *grad_g, float *grad_h, void *workspace, size_t workspace_bytes,
                              void *stream_)
{
    if (!G || !packed || !g || !h || !grad_g || !grad_h) return RB_ERR_NULL;
    const int rc = check_shape(K, out, in);
    if (rc != RB_OK) return rc;
    const int slices = (out + ROW_SLICE - 1) / ROW_SLICE;
    if (slices > 65535) return RB_ERR_SHAPE;
    if (!workspace || workspace_bytes < rb_scale_grads_workspace_bytes(K, out, in)) return RB_ERR_WORKSPACE;
    if (((uintptr_t)workspace | (uintptr_t)G) & 15) return RB_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int col_blocks = (in + 255) / 256;
    float *part_h = static_cast<float *>(workspace), *part_g = part_h + (size_t)slices * K * in;
    hipLaunchKernelGGL(grad_slab_kernel, dim3((unsigned)col_blocks, (unsigned)slices), dim3(64), 0, stream, G, packed,
                       reinterpret_cast<const __half *>(g), reinterpret_cast<const __half *>(h), K, out, in, part_h, part_g);
    hipLaunchKernelGGL(grad_finish_kernel, dim3((unsigned)((K * (in + out) + 255) / 256)), dim3(256), 0, stream, part_h,
                       slices, part_g, col_blocks, K, out, in, grad_g, grad_h);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}
