// C-ABI entry points: argument checks and kernel selection.  No allocation, no
// synchronisation; everything is enqueued on the caller's stream.
#include <hip/hip_runtime.h>

#include "rabit.h"
#include "rb_internal.h"

namespace rb {

int check_layer(const rb_layer *L)
{
    if (!L) return RB_ERR_NULL;
    if (!L->bits || !L->g || !L->h) return RB_ERR_NULL;
    if (L->K < 1 || L->K > RB_MAX_K || L->out < 1 || L->in < 32 || L->in % 32 != 0) return RB_ERR_SHAPE;
    if ((uintptr_t)L->bits & 15) return RB_ERR_ALIGN;
    if (((uintptr_t)L->g | (uintptr_t)L->h) & 1) return RB_ERR_ALIGN;
    return RB_OK;
}

}  // namespace rb

extern "C" size_t rb_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T)
{
    if (!layers || n_layers < 1 || n_ops < 1 || T < 1) return 0;
    return rb::workspace_bytes(layers, n_layers, n_ops, T);
}

extern "C" int rb_linear_gemm(const rb_layer *L, const void *X, void *Y, int T, int act_dtype,
                              int out_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = rb::check_layer(L);
    if (rc != RB_OK) return rc;
    if (!X || !Y) return RB_ERR_NULL;
    if (T < 1 || T > 65535) return RB_ERR_SHAPE;
    if (act_dtype != RB_F16 && act_dtype != RB_BF16) return RB_ERR_UNSUPPORTED;
    if (out_dtype != RB_F16 && out_dtype != RB_BF16 && out_dtype != RB_F32) return RB_ERR_UNSUPPORTED;
    if (((uintptr_t)X | (uintptr_t)Y) & 15) return RB_ERR_ALIGN;
    if (workspace_bytes < rb::workspace_bytes(L, 1, 1, T) || (workspace_bytes && !workspace))
        return RB_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15) return RB_ERR_ALIGN;
    return rb::dispatch_linear(L, X, Y, T, act_dtype, out_dtype, workspace, workspace_bytes,
                               static_cast<hipStream_t>(stream));
}

extern "C" int rb_linear_gemv(const rb_layer *L, const uint16_t *x, uint16_t *y, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    return rb_linear_gemm(L, x, y, 1, RB_F16, RB_F16, workspace, workspace_bytes, stream);
}

static int check_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                       uint16_t *const *bufs, int n_bufs, int T, void *workspace, size_t workspace_bytes);

extern "C" int rb_stack_prepare(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                                uint16_t *const *bufs, int n_bufs, int T, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    const int rc = check_stack(layers, n_layers, ops, n_ops, bufs, n_bufs, T, workspace, workspace_bytes);
    if (rc != RB_OK) return rc;
    if (!workspace) return RB_ERR_WORKSPACE;
    rb::forget_pairs(workspace);
    rb::batch::forget_plan(workspace);
    if (n_ops > 1 && rb::batch_applies(layers, n_layers, T))
        return rb::batch::prepare_plan(layers, ops, n_ops, bufs, T, workspace, workspace_bytes,
                                       static_cast<hipStream_t>(stream));
    if (T > 4)
        return rb::prepare_pairs(layers, n_layers, ops, n_ops, bufs, n_bufs, T, workspace, workspace_bytes,
                                 static_cast<hipStream_t>(stream));
    for (int n = 0; n < n_ops; ++n)
        if (!rb::mx::layer_supported(&layers[ops[n].layer], T)) return RB_ERR_UNSUPPORTED;
    return rb::mx::prepare_plan(layers, ops, n_ops, bufs, T, workspace, workspace_bytes,
                                static_cast<hipStream_t>(stream));
}

extern "C" int rb_stack_run(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return RB_ERR_NULL;
    int rc = rb::batch::launch_plan(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    if (rc != RB_ERR_UNSUPPORTED) {
        if (rc == RB_OK) rb::set_last_path(RB_PATH_BATCH);
        return rc;
    }
    rc = rb::run_pairs(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    if (rc == RB_ERR_UNSUPPORTED)
        rc = rb::mx::launch_plan(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    if (rc == RB_OK) rb::set_last_path(RB_PATH_MX);
    return rc;
}

extern "C" int rb_stack_status(const void *workspace, void *stream)
{
    if (!workspace) return RB_ERR_NULL;
    if (rb::batch::has_plan(workspace))      // no hand-over inside a launch: nothing a run could give up
        return hipStreamSynchronize(static_cast<hipStream_t>(stream)) == hipSuccess ? RB_OK : RB_ERR_HIP;
    const int rc = rb::pairs_status(workspace, static_cast<hipStream_t>(stream));
    if (rc != RB_ERR_UNSUPPORTED) return rc;
    return rb::mx::plan_status(workspace, static_cast<hipStream_t>(stream));
}

extern "C" int rb_stack_waited(const void *workspace, void *stream, unsigned long long *tiles)
{
    if (!workspace || !tiles) return RB_ERR_NULL;
    *tiles = 0;
    if (rb::batch::has_plan(workspace)) return RB_OK;
    const int rc = rb::pairs_status(workspace, static_cast<hipStream_t>(stream), tiles);
    if (rc != RB_ERR_UNSUPPORTED) return rc;
    return rb::mx::plan_status(workspace, static_cast<hipStream_t>(stream), tiles);
}

extern "C" int rb_stack_gave_up(const void *workspace, void *stream, int *reason)
{
    if (!workspace || !reason) return RB_ERR_NULL;
    *reason = 0;
    if (rb::batch::has_plan(workspace)) return RB_OK;
    const int rc = rb::pairs_status(workspace, static_cast<hipStream_t>(stream), nullptr, reason);
    if (rc != RB_ERR_UNSUPPORTED) return rc == RB_ERR_HANDOVER ? RB_OK : rc;
    const int rc2 = rb::mx::plan_status(workspace, static_cast<hipStream_t>(stream), nullptr, reason);
    return rc2 == RB_ERR_HANDOVER ? RB_OK : rc2;
}

extern "C" int rb_stack_set_option(int option, int value)
{
    if (option == RB_OPT_HANDOVER_PAUSE) {
        rb::mx::set_pause(value);
        return RB_OK;
    }
    return RB_ERR_UNSUPPORTED;
}

extern "C" int rb_stack_forget(const void *workspace)
{
    if (!workspace) return RB_ERR_NULL;
    rb::forget_pairs(workspace);
    rb::mx::forget_plan(workspace);
    rb::batch::forget_plan(workspace);
    return RB_OK;
}

extern "C" int rb_layer_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                              uint16_t *const *bufs, int n_bufs, int T, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    const int rc = check_stack(layers, n_layers, ops, n_ops, bufs, n_bufs, T, workspace, workspace_bytes);
    if (rc != RB_OK) return rc;
    return rb::dispatch_stack(layers, n_layers, ops, n_ops, bufs, n_bufs, T, workspace, workspace_bytes,
                              static_cast<hipStream_t>(stream));
}

static int check_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                       uint16_t *const *bufs, int n_bufs, int T, void *workspace, size_t workspace_bytes)
{
    if (!layers || !ops || !bufs) return RB_ERR_NULL;
    if (n_layers < 1 || n_ops < 1 || n_bufs < 1 || T < 1 || T > 65535) return RB_ERR_SHAPE;
    for (int l = 0; l < n_layers; ++l) {
        const int rc = rb::check_layer(&layers[l]);
        if (rc != RB_OK) return rc;
    }
    for (int n = 0; n < n_ops; ++n) {
        const rb_stack_op &op = ops[n];
        if (op.layer < 0 || op.layer >= n_layers || op.src < 0 || op.src >= n_bufs || op.dst < 0 ||
            op.dst >= n_bufs || op.src == op.dst)
            return RB_ERR_SHAPE;
        if (!bufs[op.src] || !bufs[op.dst]) return RB_ERR_NULL;
        if (((uintptr_t)bufs[op.src] | (uintptr_t)bufs[op.dst]) & 15) return RB_ERR_ALIGN;
    }
    if (workspace_bytes < rb::workspace_bytes(layers, n_layers, n_ops, T) || (workspace_bytes && !workspace))
        return RB_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15) return RB_ERR_ALIGN;
    return RB_OK;
}
