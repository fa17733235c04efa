// Kernel selection for one layer and for a stack of layers.
#include <hip/hip_runtime.h>

#include "rabit.h"
#include "rb_internal.h"

namespace rb {

thread_local int g_last_path = RB_PATH_NONE;
void set_last_path(int path) { g_last_path = path; }

size_t workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    if (T > 2) {
        // ops run one after the other on the caller's stream and share the scratch of the GEMM path
        size_t need = 0;
        for (int l = 0; l < n_layers; ++l)
            if (gemm::supported(&layers[l], T)) need = need > gemm::workspace_bytes(&layers[l], T) ? need : gemm::workspace_bytes(&layers[l], T);
        return need;
    }
    return mx::plan_workspace_bytes(layers, n_layers, n_ops, T);
}

int dispatch_linear(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                    void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (act_dtype == RB_F16 && out_dtype == RB_F16 && mx::layer_supported(L, T) && workspace &&
        workspace_bytes >= mx::plan_workspace_bytes(L, 1, 1, T)) {
        const rb_stack_op op{0, 0, 1};
        uint16_t *bufs[2] = {static_cast<uint16_t *>(const_cast<void *>(X)), static_cast<uint16_t *>(Y)};
        const int rc = mx::run_plan(L, &op, 1, bufs, T, workspace, workspace_bytes, stream);
        if (rc != RB_ERR_UNSUPPORTED) { g_last_path = RB_PATH_MX; return rc; }
    }
    if (T > 2 && gemm::supported(L, T) && workspace && workspace_bytes >= gemm::workspace_bytes(L, T)) {
        g_last_path = RB_PATH_GEMM;
        return gemm::launch(L, X, Y, T, act_dtype, out_dtype, workspace, stream);
    }
    g_last_path = RB_PATH_SIGNADD;
    return launch_signadd(L, X, Y, T, act_dtype, out_dtype, stream);
}

int dispatch_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                   uint16_t *const *bufs, int, int T, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    bool fused = workspace && workspace_bytes >= mx::plan_workspace_bytes(layers, n_layers, n_ops, T);
    for (int n = 0; n < n_ops && fused; ++n) fused = mx::layer_supported(&layers[ops[n].layer], T);
    if (fused) {
        const int rc = mx::run_plan(layers, ops, n_ops, bufs, T, workspace, workspace_bytes, stream);
        if (rc != RB_ERR_UNSUPPORTED) { g_last_path = RB_PATH_MX; return rc; }
    }
    for (int n = 0; n < n_ops; ++n) {
        const rb_layer *L = &layers[ops[n].layer];
        const int rc = dispatch_linear(L, bufs[ops[n].src], bufs[ops[n].dst], T, RB_F16, RB_F16, workspace,
                                       workspace_bytes, stream);
        if (rc != RB_OK) return rc;
    }
    return RB_OK;
}

}  // namespace rb

extern "C" int rb_last_path(void) { return rb::g_last_path; }
