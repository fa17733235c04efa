// rb_linear_gemm for callers that cannot provide a workspace and must not allocate: the scratch
// memory of the many-token kernel (the scaled input of both paths and the partial sums of a split
// contraction) lives in a device array of this library instead of a caller's buffer.
#include <hip/hip_runtime.h>

#include <mutex>

#include "rabit.h"
#include "rb_internal.h"

namespace {

constexpr size_t SCRATCH_BYTES = RB_NOALLOC_SCRATCH_BYTES;
// One copy per GPU that loads the library, held until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress; kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void *g_scratch_of[MAX_DEVICES] = {};      // device address of `scratch` on each device, once known

// address of the current device's copy of the array (null + status on failure)
int scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return RB_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_lock);
    if (!g_scratch_of[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RB_ERR_HIP;
        g_scratch_of[dev] = p;
    }
    *ptr = g_scratch_of[dev];
    return RB_OK;
}

}  // namespace

extern "C" size_t rb_noalloc_scratch_bytes(void) { return SCRATCH_BYTES; }

extern "C" int rb_linear_gemm_noalloc(const rb_layer *L, const void *X, void *Y, int T, int act_dtype,
                                      int out_dtype, void *stream_)
{
    const int rc = rb::check_layer(L);
    if (rc != RB_OK) return rc;
    if (!X || !Y) return RB_ERR_NULL;
    if (T < 1 || T > 65535) return RB_ERR_SHAPE;
    if (act_dtype != RB_F16 && act_dtype != RB_BF16) return RB_ERR_UNSUPPORTED;
    if (out_dtype != RB_F16 && out_dtype != RB_BF16 && out_dtype != RB_F32) return RB_ERR_UNSUPPORTED;
    if (((uintptr_t)X | (uintptr_t)Y) & 15) return RB_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // one fp16 token, two paths: the single-launch decode kernel keeps everything in LDS
    if (act_dtype == RB_F16 && out_dtype == RB_F16 && rb::gemv1::supported(L, T)) {
        rb::set_last_path(RB_PATH_MX);
        return rb::gemv1::launch(L, X, Y, stream);
    }
    // three paths at up to 32 tokens: the generic kernel, which needs no scratch memory, serves
    // whatever the many-token kernel's scratch would not fit
    const bool generic_instead = L->K == 3 && T <= 32 && rb::gemm::workspace_bytes(L, T) > SCRATCH_BYTES;
    if (rb::single_gemm_applies(L, T) && !generic_instead) {
        // the only kernels here that need scratch memory: every byte of it that they read in a
        // call they have written earlier in the same call, so nothing has to be cleared
        if (rb::gemm::workspace_bytes(L, T) > SCRATCH_BYTES) return RB_ERR_WORKSPACE;
        void *ptr = nullptr;
        const int rs = scratch_of_current_device(&ptr);
        if (rs != RB_OK) return rs;
        rb::set_last_path(RB_PATH_GEMM);
        return rb::gemm::launch(L, X, Y, T, act_dtype, out_dtype, ptr, stream);
    }
    rb::set_last_path(RB_PATH_SIGNADD);
    return rb::launch_signadd(L, X, Y, T, act_dtype, out_dtype, stream);
}
