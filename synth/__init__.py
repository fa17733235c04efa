"""Seeded synthetic inputs for the residual-binary linear layer.

This module only draws random numbers and lists shapes.  It contains none of
the layer's arithmetic (no packing, no scaling, no sign derivation, no
matrix product), so both the CPU oracle's tests and the HIP path's tests can
take their inputs from it without sharing any of the method between them.

Shapes follow the paper's inference table (Llama2-7B q_proj 4096x4096 and
gate_proj 11008x4096, Llama2-13B q_proj 5120x5120 and gate_proj 13824x5120);
the value distributions are the stand-ins for real model weights and
activations, which are not available here.
"""
from .workloads import (  # noqa: F401
    SEED_BASE,
    child_rng,
    uniform_signs,
    halfnormal_scales,
    gaussian_activations,
    outlier_activations,
    gaussian_weight,
    StackOp,
    llama_stack,
    llama_block_stack,
    LLAMA_SHAPES,
    single_layer_config,
    prefill_shapes,
)
