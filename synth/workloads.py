"""Random draws and shape lists only; see the package docstring."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

SEED_BASE = 20260205

# (d_model, d_ffn, n_layers) of the Llama-shaped stacks used as workloads.
LLAMA_SHAPES = {
    "7b": (4096, 11008, 32),
    "13b": (5120, 13824, 40),
}


def child_rng(config: int, *keys: int) -> np.random.Generator:
    """Independent generator for (config, layer, matrix, tensor, ...)."""
    return np.random.default_rng([SEED_BASE, int(config), *[int(k) for k in keys]])


def uniform_signs(rng: np.random.Generator, K: int, out: int, inn: int) -> np.ndarray:
    """i.i.d. uniform +1/-1 entries, int8 [K][out][in]."""
    bits = rng.integers(0, 2, size=(K, out, inn), dtype=np.int8)
    return (1 - 2 * bits).astype(np.int8)


def halfnormal_scales(rng: np.random.Generator, K: int, n: int,
                      sigma: float = 0.02, path_decay: float = 0.3) -> np.ndarray:
    """fp16 [K][n]: |N(0,1)|*sigma for path 1, each later path times path_decay."""
    s = np.abs(rng.standard_normal((K, n))) * sigma
    for k in range(1, K):
        s[k] *= path_decay ** k
    return s.astype(np.float16)


def gaussian_activations(rng: np.random.Generator, T: int, inn: int) -> np.ndarray:
    """fp16 [T][in] ~ N(0,1)."""
    return rng.standard_normal((T, inn)).astype(np.float16)


def outlier_activations(rng: np.random.Generator, T: int, inn: int,
                        frac: float = 0.01, gain: float = 20.0) -> np.ndarray:
    """fp16 [T][in] ~ N(0,1) with ceil(frac*in) channels (same for every token) times gain."""
    x = rng.standard_normal((T, inn))
    n_out = int(np.ceil(frac * inn))
    ch = rng.choice(inn, size=n_out, replace=False)
    x[:, ch] *= gain
    return x.astype(np.float16)


def gaussian_weight(rng: np.random.Generator, out: int, inn: int, std: float = 0.02) -> np.ndarray:
    """Full-precision stand-in weight, float64 [out][in] ~ N(0, std^2)."""
    return rng.standard_normal((out, inn)) * std


@dataclass(frozen=True)
class StackOp:
    """One linear layer of a stack: reads buffer `src`, writes buffer `dst`."""
    name: str
    out: int
    inn: int
    src: int
    dst: int


def llama_stack(which: str, n_layers: int | None = None) -> Tuple[List[StackOp], List[int]]:
    """Dependency chain made only of the linear layers of a Llama-shaped decoder.

    Per block: q, k, v read the block input; o reads v's output; gate and up
    read o's output; down reads gate's output and produces the next block's
    input.  Returns (ops in issue order, width of every buffer); buffer 0 is
    the stack input and every op writes a buffer of its own.
    """
    d, f, L = LLAMA_SHAPES[which]
    if n_layers is not None:
        L = n_layers
    ops: List[StackOp] = []
    widths: List[int] = [d]
    x = 0

    def new_buf(w: int) -> int:
        widths.append(w)
        return len(widths) - 1

    for l in range(L):
        q = new_buf(d); ops.append(StackOp(f"l{l}.q", d, d, x, q))
        k = new_buf(d); ops.append(StackOp(f"l{l}.k", d, d, x, k))
        v = new_buf(d); ops.append(StackOp(f"l{l}.v", d, d, x, v))
        o = new_buf(d); ops.append(StackOp(f"l{l}.o", d, d, v, o))
        g = new_buf(f); ops.append(StackOp(f"l{l}.gate", f, d, o, g))
        u = new_buf(f); ops.append(StackOp(f"l{l}.up", f, d, o, u))
        dn = new_buf(d); ops.append(StackOp(f"l{l}.down", d, f, g, dn))
        x = dn
    return ops, widths


def single_layer_config() -> Tuple[int, int, int]:
    """(out, in, K) of the small single-layer case."""
    return 2048, 2048, 2


def prefill_shapes() -> List[Tuple[str, int, int]]:
    """70B-shaped MLP matrices for the prefill case: (name, out, in)."""
    return [("gate", 28672, 8192), ("down", 8192, 28672)]
