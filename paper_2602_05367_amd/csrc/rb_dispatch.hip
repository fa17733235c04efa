// Kernel selection for one layer and for a stack of layers.
#include <hip/hip_runtime.h>

#include "rabit.h"
#include "rb_internal.h"

namespace rb {

size_t workspace_bytes(const rb_layer *, int, int) { return 0; }

int dispatch_linear(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                    void *, size_t, hipStream_t stream)
{
    return launch_signadd(L, X, Y, T, act_dtype, out_dtype, stream);
}

int dispatch_stack(const rb_layer *layers, int, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs,
                   int, int T, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer *L = &layers[ops[n].layer];
        const int rc = dispatch_linear(L, bufs[ops[n].src], bufs[ops[n].dst], T, RB_F16, RB_F16, workspace,
                                       workspace_bytes, stream);
        if (rc != RB_OK) return rc;
    }
    return RB_OK;
}

}  // namespace rb
