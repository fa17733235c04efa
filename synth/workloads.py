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


@dataclass(frozen=True)
class BlockOp:
    """One op of a decoder block: layer `layer` between buffers `src` and `dst`; `norm` >= 0: the
    input is normalised with that weight vector first; `epilogue` 0: nothing, 1: buffer `aux` is
    added, 2: the op is gate-times-up and `aux` is the layer of the up projection."""
    name: str
    layer: int
    src: int
    dst: int
    norm: int
    epilogue: int
    aux: int


def llama_block_stack(which: str, n_layers: int, in_place: bool = False
                      ) -> Tuple[List[BlockOp], List[Tuple[str, int, int]], List[int], List[int]]:
    """The linear layers of a Llama-shaped decoder with what sits between them, attention left out.

    Per block: q, k, v read the normalised block input x; o reads v's output and x is added to it;
    gate and up read the normalised result x1, silu(gate) * up feeds down, and x1 is added to
    down's output, which is the next block's input.  Returns (ops in issue order, (name, out, in)
    of every layer, width of every buffer, width of every norm weight); buffer 0 is the stack
    input.  Every op writes a buffer of its own unless `in_place`, where the residual stream lives
    in buffer 0 throughout.
    """
    d, f, _ = LLAMA_SHAPES[which]
    ops: List[BlockOp] = []
    shapes: List[Tuple[str, int, int]] = []
    widths: List[int] = [d]
    norms: List[int] = []
    x = 0

    def new_buf(w: int) -> int:
        widths.append(w)
        return len(widths) - 1

    def new_layer(name: str, out: int, inn: int) -> int:
        shapes.append((name, out, inn))
        return len(shapes) - 1

    for l in range(n_layers):
        n1, n2 = len(norms), len(norms) + 1
        norms += [d, d]
        for name in ("q", "k"):
            ops.append(BlockOp(f"l{l}.{name}", new_layer(f"l{l}.{name}", d, d), x, new_buf(d), n1, 0, -1))
        v = new_buf(d)
        ops.append(BlockOp(f"l{l}.v", new_layer(f"l{l}.v", d, d), x, v, n1, 0, -1))
        x1 = x if in_place else new_buf(d)
        ops.append(BlockOp(f"l{l}.o", new_layer(f"l{l}.o", d, d), v, x1, -1, 1, x))
        gate, up = new_layer(f"l{l}.gate", f, d), new_layer(f"l{l}.up", f, d)
        act = new_buf(f)
        ops.append(BlockOp(f"l{l}.gate_up", gate, x1, act, n2, 2, up))
        x2 = x1 if in_place else new_buf(d)
        ops.append(BlockOp(f"l{l}.down", new_layer(f"l{l}.down", d, f), act, x2, -1, 1, x1))
        x = x2
    return ops, shapes, widths, norms


def single_layer_config() -> Tuple[int, int, int]:
    """(out, in, K) of the small single-layer case."""
    return 2048, 2048, 2


def prefill_shapes() -> List[Tuple[str, int, int]]:
    """70B-shaped MLP matrices for the prefill case: (name, out, in)."""
    return [("gate", 28672, 8192), ("down", 8192, 28672)]
