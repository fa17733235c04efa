// Declarations shared between the entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>

#include "rabit.h"

namespace rb {

int check_layer(const rb_layer *L);
void set_last_path(int path);

// generic sign-XOR + add kernel, any supported shape, T via grid.y
int launch_signadd(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                   hipStream_t stream);

size_t workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);
// stacks that run on the small-batch kernel (see rb_dispatch.hip)
bool batch_applies(const rb_layer *layers, int n_layers, int T);
// a single call of T tokens on this layer takes the many-token kernel (given the scratch memory it needs)
bool single_gemm_applies(const rb_layer *L, int T);

int dispatch_linear(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype,
                    void *workspace, size_t workspace_bytes, hipStream_t stream);

int dispatch_stack(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops,
                   uint16_t *const *bufs, int n_bufs, int T, void *workspace, size_t workspace_bytes,
                   hipStream_t stream);

// stacks of 5..7 tokens as passes of the fused kernel over groups of four tokens: one plan per pass
// in consecutive parts of the workspace (RB_ERR_UNSUPPORTED where that does not apply)
int prepare_pairs(const rb_layer *layers, int n_layers, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs,
                  int n_bufs, int T, void *workspace, size_t workspace_bytes, hipStream_t stream);
int run_pairs(void *workspace, size_t workspace_bytes, hipStream_t stream);
void forget_pairs(const void *workspace);
int pairs_status(const void *workspace, hipStream_t stream, unsigned long long *waited = nullptr, int *reason = nullptr);     // RB_ERR_UNSUPPORTED: no plans of this kind

namespace gemm {
// many-token matrix-core GEMM (K = 2): workspace holds the scaled input of both paths
bool supported(const rb_layer *L, int T);
size_t workspace_bytes(const rb_layer *L, int T);
int launch(const rb_layer *L, const void *X, void *Y, int T, int act_dtype, int out_dtype, void *workspace,
           hipStream_t stream);
}  // namespace gemm

namespace gemv1 {
// one layer, one token, one launch, nothing prepared (K = 2; the expanded input must fit in LDS);
// same bits as the op would give inside a stack
bool supported(const rb_layer *L, int T);
int launch(const rb_layer *L, const void *x, void *y, hipStream_t stream);
}  // namespace gemv1

namespace batch {
// small-batch path (K = 2 or 3, up to 16 tokens): every op streams its weights once for all
// tokens; independent ops share a launch, dependent ones are ordered by the stream
bool layer_supported(const rb_layer *L, int T);
size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);
int prepare_plan(const rb_layer *layers, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs, int T,
                 void *workspace, size_t workspace_bytes, hipStream_t stream);
int launch_plan(void *workspace, size_t workspace_bytes, hipStream_t stream);      // RB_ERR_UNSUPPORTED: no plan of this kind
bool has_plan(const void *workspace);
void forget_plan(const void *workspace);
}  // namespace batch

namespace mx {
// workgroups of the decode kernels: one per compute unit of the current device (0: no device)
int device_groups();
// matrix-core path (K = 2 and T <= 4, or K = 3 and T = 1): whole op lists run as one persistent kernel
bool layer_supported(const rb_layer *L, int T);
size_t plan_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);
int run_plan(const rb_layer *layers, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs, int T,
             void *workspace, size_t workspace_bytes, hipStream_t stream);
// the two halves of run_plan: set-up that depends only on the frozen layers and the buffer
// addresses, and the per-token launch
int prepare_plan(const rb_layer *layers, const rb_stack_op *ops, int n_ops, uint16_t *const *bufs, int T,
                 void *workspace, size_t workspace_bytes, hipStream_t stream);
int launch_plan(void *workspace, size_t workspace_bytes, hipStream_t stream);
void forget_plan(const void *workspace);
// decoder blocks (norms, gate times up, residual additions in the kernel's finishing step); run,
// checked and forgotten like any other plan of this kernel
size_t block_workspace_bytes(const rb_layer *layers, int n_layers, int n_ops, int T);
int prepare_block(const rb_layer *layers, const uint16_t *const *norm_w, float eps, const rb_block_op *ops, int n_ops,
                  uint16_t *const *bufs, int T, void *workspace, size_t workspace_bytes, hipStream_t stream);
// waits for the stream; RB_ERR_HANDOVER if a run of this plan gave up a wait, RB_ERR_WORKSPACE: no plan
// waited (optional): += input tiles that compute wavefronts found not yet written and waited for, since the plan was made
int plan_status(const void *workspace, hipStream_t stream, unsigned long long *waited = nullptr, int *reason = nullptr);
// pause between a workgroup's last stores of a stage and the moment its compute wavefronts ask for
// that stage's outputs, in clocks (< 0: the built-in timing); launches made afterwards use it
void set_pause(int clks);
}  // namespace mx

}  // namespace rb
