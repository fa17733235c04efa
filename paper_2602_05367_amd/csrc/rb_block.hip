// The decoder block around the residual-binary layers (the end-to-end decoding setting of
// Section 5.4 and the inference table: a Llama-2 block): entry points of the fused form, which
// runs on the persistent decode kernel, and the three operations as kernels of their own for
// callers that run a block op by op.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "rabit.h"
#include "rb_internal.h"

namespace rb {
namespace {

// y = x / sqrt(mean_j x_j^2 + eps) (.) w, one workgroup per token; fp32 arithmetic, fp16 in and out
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __half *x, const __half *w, __half *y, int n, float eps)
{
    const __half *xr = x + (size_t)blockIdx.x * n;
    __half *yr = y + (size_t)blockIdx.x * n;
    float sum = 0.f;
    for (int j = threadIdx.x; j < n; j += 256) {
        const float v = __half2float(xr[j]);
        sum += v * v;
    }
    __shared__ float red[256];
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const float rinv = rsqrtf(red[0] / (float)n + eps);
    for (int j = threadIdx.x; j < n; j += 256) yr[j] = __float2half_rn(__half2float(xr[j]) * rinv * __half2float(w[j]));
}

// y = silu(a) * b, elementwise
__global__ __launch_bounds__(256) void silu_mul_kernel(const __half *a, const __half *b, __half *y, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = __half2float(a[i]);
    y[i] = __float2half_rn(g / (1.f + __expf(-g)) * __half2float(b[i]));
}

__global__ __launch_bounds__(256) void add_kernel(const __half *a, const __half *b, __half *y, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    y[i] = __float2half_rn(__half2float(a[i]) + __half2float(b[i]));
}

int check_block(const rb_layer *layers, int n_layers, const uint16_t *const *norm_weights, int n_norms, float eps,
                const rb_block_op *ops, int n_ops, uint16_t *const *bufs, int n_bufs, int T, void *workspace,
                size_t workspace_bytes)
{
    if (!layers || !ops || !bufs || (n_norms > 0 && !norm_weights)) return RB_ERR_NULL;
    if (n_layers < 1 || n_ops < 1 || n_bufs < 1 || n_norms < 0 || T < 1 || !(eps >= 0.f)) return RB_ERR_SHAPE;
    for (int l = 0; l < n_layers; ++l) {
        const int rc = check_layer(&layers[l]);
        if (rc != RB_OK) return rc;
    }
    for (int i = 0; i < n_norms; ++i) {
        if (!norm_weights[i]) return RB_ERR_NULL;
        if ((uintptr_t)norm_weights[i] & 1) return RB_ERR_ALIGN;
    }
    for (int n = 0; n < n_ops; ++n) {
        const rb_block_op &op = ops[n];
        if (op.layer < 0 || op.layer >= n_layers || op.src < 0 || op.src >= n_bufs || op.dst < 0 || op.dst >= n_bufs ||
            op.src == op.dst || op.norm < -1 || op.norm >= n_norms)
            return RB_ERR_SHAPE;
        if (!bufs[op.src] || !bufs[op.dst]) return RB_ERR_NULL;
        if (((uintptr_t)bufs[op.src] | (uintptr_t)bufs[op.dst]) & 15) return RB_ERR_ALIGN;
        if (op.epilogue == RB_EPI_ADD) {
            if (op.aux < 0 || op.aux >= n_bufs || op.aux == op.src) return RB_ERR_SHAPE;
            if (!bufs[op.aux]) return RB_ERR_NULL;
            if ((uintptr_t)bufs[op.aux] & 15) return RB_ERR_ALIGN;
        } else if (op.epilogue == RB_EPI_SILU_MUL) {
            if (op.aux < 0 || op.aux >= n_layers) return RB_ERR_SHAPE;
            const rb_layer &a = layers[op.layer], &b = layers[op.aux];
            if (a.out != b.out || a.in != b.in || a.K != b.K) return RB_ERR_SHAPE;
        } else if (op.epilogue != RB_EPI_NONE) {
            return RB_ERR_SHAPE;
        }
    }
    if (workspace_bytes < mx::block_workspace_bytes(layers, n_layers, n_ops, T) || !workspace) return RB_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15) return RB_ERR_ALIGN;
    return RB_OK;
}

}  // namespace
}  // namespace rb

extern "C" size_t rb_block_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    if (!layers || n_layers < 1 || n_ops < 1 || T < 1) return 0;
    return rb::mx::block_workspace_bytes(layers, n_layers, n_ops, T);
}

extern "C" int rb_block_prepare(const rb_layer *layers, int n_layers, const uint16_t *const *norm_weights, int n_norms,
                                float eps, const rb_block_op *ops, int n_ops, uint16_t *const *bufs, int n_bufs, int T,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = rb::check_block(layers, n_layers, norm_weights, n_norms, eps, ops, n_ops, bufs, n_bufs, T, workspace,
                                   workspace_bytes);
    if (rc != RB_OK) return rc;
    rb_stack_forget(workspace);
    return rb::mx::prepare_block(layers, norm_weights, eps, ops, n_ops, bufs, T, workspace, workspace_bytes,
                                 static_cast<hipStream_t>(stream));
}

extern "C" int rb_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int T, int n, float eps, void *stream)
{
    if (!x || !w || !y) return RB_ERR_NULL;
    if (T < 1 || T > 65535 || n < 1 || !(eps >= 0.f)) return RB_ERR_SHAPE;
    hipLaunchKernelGGL(rb::rmsnorm_kernel, dim3(T), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const __half *>(x), reinterpret_cast<const __half *>(w),
                       reinterpret_cast<__half *>(y), n, eps);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

extern "C" int rb_silu_mul(const uint16_t *gate, const uint16_t *up, uint16_t *y, size_t n, void *stream)
{
    if (!gate || !up || !y) return RB_ERR_NULL;
    if (n < 1 || n > ((size_t)1 << 38)) return RB_ERR_SHAPE;
    hipLaunchKernelGGL(rb::silu_mul_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const __half *>(gate), reinterpret_cast<const __half *>(up),
                       reinterpret_cast<__half *>(y), n);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}

extern "C" int rb_add(const uint16_t *a, const uint16_t *b, uint16_t *y, size_t n, void *stream)
{
    if (!a || !b || !y) return RB_ERR_NULL;
    if (n < 1 || n > ((size_t)1 << 38)) return RB_ERR_SHAPE;
    hipLaunchKernelGGL(rb::add_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const __half *>(a), reinterpret_cast<const __half *>(b),
                       reinterpret_cast<__half *>(y), n);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_ERR_HIP;
}
