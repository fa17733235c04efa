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

// One wavefront per row and chunk of COUPLE_CHUNK columns; a step covers 64 consecutive columns,
// lane l holding column 64 m + l, so that a ballot of "residual is negative" is two canonical words at once (bit b = column 32 w + b,
// 1 means -1).  The residual is fp32 with one rounding for g * h and one for the subtraction, the
// arithmetic the definition fixes (the sign of the product is exact).
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
    const int chunk0 = blockIdx.y * COUPLE_CHUNK, chunk1 = min(in, chunk0 + COUPLE_CHUNK);
    // the chunk's weights first, all loads in flight at once: a wavefront that asked for them one
    // step at a time would spend its life waiting for memory
    float wv[COUPLE_CHUNK / 64];
#pragma unroll
    for (int i = 0; i < COUPLE_CHUNK / 64; ++i) {
        const int c = chunk0 + 64 * i + lane;
        wv[i] = c < in ? W[(size_t)row * in + c] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < COUPLE_CHUNK / 64; ++i) {
        const int c0 = chunk0 + 64 * i;
        if (c0 >= chunk1) break;
        const int c = c0 + lane;
        const bool real = c < in;
        float r = wv[i];
        for (int k = 0; k < K; ++k) {
            const bool neg = real && !(r >= 0.f);                 // sign(0) = +1; columns past the end read as +1
            const unsigned long long bal = __ballot(neg);
            const float prod = __fmul_rn(gr[k], real ? __half2float(h[(size_t)k * in + c]) : 0.f);
            r = neg ? __fadd_rn(r, prod) : __fsub_rn(r, prod);
            const int w = (c0 >> 5) + (lane >> 5);                // the word this half of the wavefront covers
            const uint32_t word = lane < 32 ? (uint32_t)bal : (uint32_t)(bal >> 32);
            if (packed && (lane & 31) == 0 && w < W32) packed[((size_t)k * out + row) * W32 + w] = word;
            if (native) {
                // native bit p of a word is column 8 (p % 4) + p / 4: every lane supplies one bit
                const int p = lane & 31;
                const unsigned long long nat = __ballot((word >> column_of_native_bit(p)) & 1u);
                const uint32_t nword = lane < 32 ? (uint32_t)nat : (uint32_t)(nat >> 32);
                if ((lane & 31) == 0 && w < W32) {
                    const int rt = row / TILE_ROWS, ct = w / 8, cc = (w % 8) / 4, q = w % 4;
                    native[((size_t)rt * CT + ct) * tile_words(K) + lane_word((row % TILE_ROWS) + 16 * q, cc, k, K)] = nword;
                }
            }
        }
        if (residual && real) residual[(size_t)row * in + c] = r;
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

// grad g: one wavefront per row; a lane takes four consecutive columns at a time (one 16-byte load
// of G, four bits of one sign word per path), four such steps in flight; K sums per lane, then a
// butterfly over the wavefront (a fixed order for a given width).
__global__ __launch_bounds__(256) void grad_rows_kernel(const float *__restrict__ G, const uint32_t *__restrict__ packed,
                                                        const __half *__restrict__ h, int K, int out, int in,
                                                        float *__restrict__ grad_g)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= out) return;
    const int W32 = in / 32;
    const float4 *Grow = reinterpret_cast<const float4 *>(G + (size_t)row * in);     // in % 32 == 0: 16-byte aligned rows
    float s[RB_MAX_K] = {0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < in; c0 += 4 * 256) {
        float4 gv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 256 * u + 4 * lane;
            gv[u] = c < in ? Grow[c >> 2] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 256 * u + 4 * lane;
            if (c < in) {
                const float v[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                for (int k = 0; k < K; ++k) {
                    const uint32_t bits4 = packed[((size_t)k * out + row) * W32 + (c >> 5)] >> (c & 31);
                    const __half *hk = h + (size_t)k * in + c;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = __half2float(hk[e]) * v[e];
                        s[k] += (bits4 >> e) & 1u ? -t : t;
                    }
                }
            }
        }
    }
    for (int k = 0; k < K; ++k) {
        float v = s[k];
        for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d);
        if (lane == 0) grad_g[(size_t)k * out + row] = v;
    }
}

// grad h, first pass: a thread takes four consecutive columns and walks the ROW_SLICE rows of its
// slice in order, eight rows in flight; partial sums [slice][K][in].  Second pass: the slices are
// added in order.
__global__ __launch_bounds__(64) void grad_cols_kernel(const float *__restrict__ G, const uint32_t *__restrict__ packed,
                                                       const __half *__restrict__ g, int K, int out, int in,
                                                       float *__restrict__ part)
{
    const int c = (blockIdx.x * 64 + threadIdx.x) * 4, slice = blockIdx.y;
    if (c >= in) return;
    const int W32 = in / 32, r0 = slice * ROW_SLICE, r1 = min(out, r0 + ROW_SLICE);
    float s[RB_MAX_K][4];
    for (int k = 0; k < RB_MAX_K; ++k)
        for (int e = 0; e < 4; ++e) s[k][e] = 0.f;
    for (int rb = r0; rb < r1; rb += 8) {
        float4 gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            gv[u] = rb + u < r1 ? *reinterpret_cast<const float4 *>(G + (size_t)(rb + u) * in + c) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = rb + u;
            if (r < r1) {
                const float v[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                for (int k = 0; k < K; ++k) {
                    const uint32_t bits4 = packed[((size_t)k * out + r) * W32 + (c >> 5)] >> (c & 31);
                    const float gk = __half2float(g[(size_t)k * out + r]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = gk * v[e];
                        s[k][e] += (bits4 >> e) & 1u ? -t : t;
                    }
                }
            }
        }
    }
    for (int k = 0; k < K; ++k)
        *reinterpret_cast<float4 *>(part + ((size_t)slice * K + k) * in + c) = make_float4(s[k][0], s[k][1], s[k][2], s[k][3]);
}

__global__ __launch_bounds__(256) void grad_cols_finish_kernel(const float *__restrict__ part, int slices, int K, int in,
                                                               float *__restrict__ grad_h)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= K * in) return;
    float s = 0.f;
    for (int sl = 0; sl < slices; ++sl) s += part[(size_t)sl * K * in + i];
    grad_h[i] = s;
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
    if (((uintptr_t)W | (uintptr_t)packed | (uintptr_t)native | (uintptr_t)residual) & 3) return RB_ERR_ALIGN;
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
    return (size_t)((out + ROW_SLICE - 1) / ROW_SLICE) * K * in * sizeof(float);
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
    hipLaunchKernelGGL(grad_rows_kernel, dim3((unsigned)((out + 3) / 4)), dim3(256), 0, stream, G, packed,
                       reinterpret_cast<const __half *>(h), K, out, in, grad_g);
    hipLaunchKernelGGL(grad_cols_kernel, dim3((unsigned)((in + 255) / 256), (unsigned)slices), dim3(64), 0, stream, G,
                       packed, reinterpret_cast<const __half *>(g), K, out, in, static_cast<float *>(workspace));
    hipLaunchKernelGGL(grad_cols_finish_kernel, dim3((unsigned)((K * in + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const float *>(workspace), slices, K, in, grad_h);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}
