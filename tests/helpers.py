"""Shared by the GPU parity tests: build a device layer and its oracle inputs."""
import numpy as np
import torch

import oracle
import synth
import paper_2602_05367_amd as rb

TOL = 1e-3   # max per-vector relative L2 error vs the fp64 oracle (fp16 in/out, fp32 accumulate)


def random_layer(rng, K, out, inn, gain=1.0):
    """Uniform +-1 signs and half-normal fp16 scales (the small-config recipe)."""
    signs = synth.uniform_signs(rng, K, out, inn)
    g = (synth.halfnormal_scales(rng, K, out).astype(np.float64) * gain).astype(np.float16)
    h = synth.halfnormal_scales(rng, K, inn)
    return signs, g, h


def to_device_layer(signs, g, h):
    return rb.Layer.from_host(signs, g, h)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """torch bf16 tensor -> uint16 bit patterns (numpy has no bf16)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def max_rel_l2(y_gpu: torch.Tensor, ref: np.ndarray) -> float:
    if y_gpu.dtype == torch.bfloat16:
        got = oracle.bf16_bits_to_f64(bf16_bits(y_gpu)).reshape(ref.shape)
    else:
        got = y_gpu.detach().cpu().numpy().astype(np.float64).reshape(ref.shape)
    return float(oracle.relative_l2(got, ref).max())


def build_stack(which, n_layers, config, T, derived, shrink=None, outliers=False, gain=1.0):
    """Host-side description of a Llama-shaped stack: per op (signs, g, h) and the
    buffer list.  `derived`: paths come from a Gaussian W through the oracle's
    derivation, and each op's g carries a constant that brings its free-running
    output to RMS ~1 (a pure rescale of a stored parameter, so that 100+ dependent
    ops stay inside the fp16 range).  `shrink` maps real widths to small ones."""
    ops, widths = synth.llama_stack(which, n_layers)
    m = (lambda w: shrink.get(w, w)) if shrink else (lambda w: w)
    widths = [m(w) for w in widths]
    rng0 = synth.child_rng(config, 0)
    bufs = [None] * len(widths)
    bufs[0] = (synth.outlier_activations if outliers else synth.gaussian_activations)(rng0, T, widths[0])
    layers = []
    for n, op in enumerate(ops):
        rng = synth.child_rng(config, 1, n)
        out, inn = m(op.out), m(op.inn)
        if derived:
            signs, g, h, _ = oracle.derive(synth.gaussian_weight(rng, out, inn), 2)
            y = oracle.forward(signs, g, h, bufs[op.src])
            c = 1.0 / np.sqrt((y ** 2).mean())
            g = (g.astype(np.float64) * c).astype(np.float16)
        else:
            signs, g, h = random_layer(rng, 2, out, inn, gain=gain)
        layers.append((signs, g, h))
        bufs[op.dst] = oracle.forward(signs, g, h, bufs[op.src]).astype(np.float16)
    return ops, widths, layers, bufs
