"""Residual-binary linear layer (RaBiT inference path) for AMD MI355X.

The product is ``librabit.so`` (hand-written HIP for gfx950, C ABI declared in
``include/rabit.h``); this package is its ctypes binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import (  # noqa: F401
    Layer, Stack, RabitError, lib, LIB_PATH, EXPORTS,
    rb_pack, rb_unpack, rb_native_bytes, rb_repack_native, rb_unpack_native,
    rb_linear_gemv, rb_linear_gemm, rb_layer_stack, rb_workspace_bytes,
    rb_linear_gemm_noalloc, rb_noalloc_scratch_bytes, rb_stack_set_option, RB_OPT_HANDOVER_PAUSE,
    rb_couple, rb_weight_grad, rb_scale_grads,
    rb_derive_iterative, Block, rb_rmsnorm, rb_silu_mul, rb_add, RB_EPI_NONE, RB_EPI_ADD, RB_EPI_SILU_MUL,
    rb_dense_gemv_f16, rb_stream_read, rb_version, rb_last_path,
    RB_PATH_NONE, RB_PATH_SIGNADD, RB_PATH_MX, RB_PATH_GEMM, RB_PATH_BATCH,
    RB_OK, RB_ERR_NULL, RB_ERR_SHAPE, RB_ERR_ALIGN, RB_ERR_UNSUPPORTED, RB_ERR_HIP,
    RB_ERR_WORKSPACE, RB_ERR_VALUE, RB_ERR_HANDOVER, RB_F16, RB_BF16, RB_F32,
)
