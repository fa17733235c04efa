"""CPU oracle for the residual-binary linear layer.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library
or its Python binding and never imports them.

What each function follows:

* ``pack`` / ``unpack``      - appendix "Weight Packing" (32 columns per word,
                               +1 -> 0, -1 -> 1; least-significant bit = lowest
                               column is this build's reading).
* ``effective_weight``       - Section 4.1 and Eq. (stacked binary weight).
* ``forward``                - Alg. 2 "compute layer output", Y = W_hat X.
* ``svid`` / ``derive``      - Section 4.2 steps 1-3 and Alg. 2 forward loop for
                               the signs; Section 4.3 (SVID: rank-1 SVD of the
                               magnitudes) for the scales, one greedy pass.
* ``precondition`` / ``derive_iterative``
                             - Section 4.3 Eq. (init-iter), Eq. (init-calib) and
                               Alg. 1: Gauss-Seidel sweeps of SVID over the
                               residuals of a preconditioned target, scales
                               mapped back to the original domain.
* ``couple``                 - Alg. 2 forward loop ("on-the-fly residual coupling")
                               with given scales, in fp32 as a training step holds
                               the shared weight.
* ``scale_grads``            - Eq. (RaBiT-grad-gh), gradients of the scales; with
                               ``weight_grad`` Eq. (RaBiT-grad-wfp).
* ``stack_forward``          - the layer applied op after op (fp16 between ops).
* ``rmsnorm`` / ``silu`` / ``block_forward``
                             - the operations that sit between the linear layers of
                               the Llama-2 decoder block the end-to-end decoding
                               figures are measured on (Section 5.4, inference
                               table): root-mean-square normalisation with a weight
                               in front of a layer, gate(x) -> SiLU, times up(x),
                               and the addition of the residual stream, each by its
                               textbook definition.

All floating point is fp64.  Stored fp16 / bf16 values are widened exactly.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rb_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C part with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
             _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i = ctypes.c_int
        p = ctypes.c_void_p
        lib.orc_pack.argtypes = [p, i, i, i, p]
        lib.orc_unpack.argtypes = [p, i, i, i, p]
        lib.orc_effective_weight.argtypes = [p, p, p, i, i, i, p]
        lib.orc_matmul.argtypes = [p, p, i, i, i, p]
        for f in (lib.orc_pack, lib.orc_unpack, lib.orc_effective_weight, lib.orc_matmul,
                  lib.orc_threads):
            f.restype = i
        _lib = lib
    return _lib


def threads() -> int:
    """Host threads the C loops use."""
    return int(_load().orc_threads())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------
# stored formats -> fp64 (exact widening)
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


# --------------------------------------------------------------------------
# Weight Packing
# --------------------------------------------------------------------------
def pack(signs: np.ndarray) -> np.ndarray:
    """int8 +1/-1 [K][out][in] -> uint32 [K][out][in/32]."""
    signs = np.ascontiguousarray(signs, dtype=np.int8)
    K, out, inn = signs.shape
    if inn % 32 != 0:
        raise ValueError("in must be a multiple of 32")
    packed = np.zeros((K, out, inn // 32), dtype=np.uint32)
    rc = _load().orc_pack(_ptr(signs), K, out, inn, _ptr(packed))
    if rc != 0:
        raise ValueError(f"orc_pack failed ({rc}): entries must be +1 or -1")
    return packed


def unpack(packed: np.ndarray) -> np.ndarray:
    """uint32 [K][out][in/32] -> int8 +1/-1 [K][out][in]."""
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    K, out, W32 = packed.shape
    signs = np.zeros((K, out, W32 * 32), dtype=np.int8)
    rc = _load().orc_unpack(_ptr(packed), K, out, W32 * 32, _ptr(signs))
    if rc != 0:
        raise ValueError(f"orc_unpack failed ({rc})")
    return signs


# --------------------------------------------------------------------------
# Forward: Section 4.1, Eq. (stacked binary weight), Alg. 2 output line
# --------------------------------------------------------------------------
def effective_weight(signs: np.ndarray, g, h) -> np.ndarray:
    """W_hat[i][j] = sum_k g_k[i] B_k[i][j] h_k[j], fp64 [out][in]."""
    signs = np.ascontiguousarray(signs, dtype=np.int8)
    K, out, inn = signs.shape
    g = _f64(g).reshape(K, out)
    h = _f64(h).reshape(K, inn)
    What = np.empty((out, inn), dtype=np.float64)
    rc = _load().orc_effective_weight(_ptr(signs), _ptr(g), _ptr(h), K, out, inn, _ptr(What))
    if rc != 0:
        raise ValueError(f"orc_effective_weight failed ({rc})")
    return What


def matmul(What: np.ndarray, X) -> np.ndarray:
    """Y[t][i] = sum_j What[i][j] X[t][j]; X [T][in] -> Y fp64 [T][out]."""
    What = _f64(What)
    out, inn = What.shape
    X = _f64(X).reshape(-1, inn)
    T = X.shape[0]
    Y = np.empty((T, out), dtype=np.float64)
    rc = _load().orc_matmul(_ptr(What), _ptr(X), out, inn, T, _ptr(Y))
    if rc != 0:
        raise ValueError(f"orc_matmul failed ({rc})")
    return Y


def forward(signs: np.ndarray, g, h, X) -> np.ndarray:
    """y = (sum_k g_k (.) B_k (.) h_k) x for every row of X.  fp64 [T][out]."""
    return matmul(effective_weight(signs, g, h), X)


def relative_l2(y_test, y_ref) -> np.ndarray:
    """Per-vector ||y_test - y_ref||_2 / ||y_ref||_2 over the last axis."""
    a = _f64(y_test)
    b = _f64(y_ref)
    a = a.reshape(-1, a.shape[-1])
    b = b.reshape(-1, b.shape[-1])
    num = np.sqrt(((a - b) ** 2).sum(axis=1))
    den = np.sqrt((b ** 2).sum(axis=1))
    return num / np.where(den == 0.0, 1.0, den)


# --------------------------------------------------------------------------
# Derivation of the paths from a full-precision weight
# --------------------------------------------------------------------------
def sign(R: np.ndarray) -> np.ndarray:
    """sign with sign(0) = +1 (the paper leaves sign(0) open; B must be +-1)."""
    return np.where(np.asarray(R) >= 0.0, 1, -1).astype(np.int8)


def leading_singular_pair(A: np.ndarray, tol: float = 1e-13, max_iter: int = 200
                          ) -> Tuple[float, np.ndarray, np.ndarray]:
    """Leading singular triplet (sigma, a, b) of a non-negative matrix A by
    power iteration from the all-ones vector; a, b have unit norm and
    non-negative entries (Perron-Frobenius)."""
    A = _f64(A)
    b = np.ones(A.shape[1]) / np.sqrt(A.shape[1])
    sigma = 0.0
    for _ in range(max_iter):
        a = A @ b
        na = np.linalg.norm(a)
        if na == 0.0:
            return 0.0, np.zeros(A.shape[0]), b
        a /= na
        b_new = A.T @ a
        s_new = np.linalg.norm(b_new)
        b_new /= s_new
        done = abs(s_new - sigma) <= tol * s_new and np.linalg.norm(b_new - b) <= 1e-10
        b, sigma = b_new, s_new
        if done:
            break
    a = A @ b
    sigma = float(np.linalg.norm(a))
    a /= sigma
    return sigma, a, b


def svid(R: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """SVID of Section 4.3: B = sign(R); (g, h) = rank-1 SVD fit of |R|,
    sigma split evenly: g = sqrt(sigma) a, h = sqrt(sigma) b.  fp64."""
    R = _f64(R)
    sigma, a, b = leading_singular_pair(np.abs(R))
    r = np.sqrt(sigma)
    return sign(R), r * a, r * b


def derive(W: np.ndarray, K: int, round_scales: bool = True):
    """Greedy derivation (Alg. 2 forward loop with scales from one SVID pass):
    R_0 = W; B_k = sign(R_{k-1}); (g_k, h_k) = SVID scales of R_{k-1};
    R_k = R_{k-1} - g_k (.) B_k (.) h_k.

    With ``round_scales`` the scales are rounded to fp16 before the residual is
    formed, so that the next path corrects what the deployed path really does.
    Returns (signs int8 [K][out][in], g [K][out], h [K][in], residual Frobenius
    norms [K+1]); g, h are float16 when rounded, float64 otherwise.
    """
    R = _f64(W).copy()
    out, inn = R.shape
    signs = np.empty((K, out, inn), dtype=np.int8)
    gs, hs = [], []
    norms = [float(np.linalg.norm(R))]
    for k in range(K):
        B, g, h = svid(R)
        if round_scales:
            g = g.astype(np.float16)
            h = h.astype(np.float16)
        signs[k] = B
        gs.append(g)
        hs.append(h)
        R = R - g.astype(np.float64)[:, None] * B.astype(np.float64) * h.astype(np.float64)[None, :]
        norms.append(float(np.linalg.norm(R)))
    return signs, np.stack(gs), np.stack(hs), np.array(norms)


def precondition(W: np.ndarray, s_in, s_out, alpha_in: float, alpha_out: float):
    """Eq. (init-calib) with the normalisation of Alg. 1 step 1: both statistics
    are divided by their maximum, then W' = s_out^a_out (.) W (.) s_in^a_in
    (s_out scales rows, s_in columns).  Returns (W', row factors, column
    factors); the factors are what step 3 divides the scales by."""
    W = _f64(W)
    s_in = _f64(s_in)
    s_out = _f64(s_out)
    if s_in.shape != (W.shape[1],) or s_out.shape != (W.shape[0],):
        raise ValueError("s_in is per input column, s_out per output row")
    if np.any(s_in <= 0.0) or np.any(s_out <= 0.0):
        raise ValueError("channel statistics must be positive")
    rows = (s_out / s_out.max()) ** alpha_out
    cols = (s_in / s_in.max()) ** alpha_in
    return rows[:, None] * W * cols[None, :], rows, cols


def derive_iterative(W: np.ndarray, K: int, T_max: int = 20, s_in=None, s_out=None,
                     alpha_in: float = 0.0, alpha_out: float = 0.0):
    """Alg. 1 (calibrated Iterative Residual SVID), fp64 throughout.

    Step 1: W' from ``precondition`` (no statistics given: W' = W).
    Step 2: W_hat_i^(0) = 0; for t = 1..T_max, for i = 1..K:
            R_i = W' - sum_{j<i} W_hat_j^(t) - sum_{j>i} W_hat_j^(t-1)   (Eq. init-iter)
            (B_i, g_i', h_i') = SVID(R_i);  W_hat_i^(t) = g_i' (.) B_i (.) h_i'.
    Step 3: g_i = g_i' / row factors, h_i = h_i' / column factors.

    Returns (signs int8 [K][out][in], g [K][out], h [K][in], err) where
    err[t][i] = || W' - sum_j W_hat_j ||_F right after path i was updated in
    sweep t (err has shape [T_max][K]; the error lives in the preconditioned
    domain, the one the iteration minimises).
    """
    if K < 1 or T_max < 1:
        raise ValueError("K >= 1 and T_max >= 1")
    W = _f64(W)
    if s_in is None and s_out is None:
        Wp, rows, cols = W.copy(), np.ones(W.shape[0]), np.ones(W.shape[1])
    else:
        Wp, rows, cols = precondition(W, s_in, s_out, alpha_in, alpha_out)
    out, inn = Wp.shape
    signs = np.ones((K, out, inn), dtype=np.int8)
    g = np.zeros((K, out))
    h = np.zeros((K, inn))
    What = np.zeros((K, out, inn))
    err = np.empty((T_max, K))
    for t in range(T_max):
        for i in range(K):
            # paths j < i were already replaced in this sweep, paths j > i still hold sweep t - 1
            R = Wp - (What.sum(axis=0) - What[i])
            signs[i], g[i], h[i] = svid(R)
            What[i] = g[i][:, None] * signs[i].astype(np.float64) * h[i][None, :]
            err[t, i] = float(np.linalg.norm(Wp - What.sum(axis=0)))
    return signs, g / rows[None, :], h / cols[None, :], err


# --------------------------------------------------------------------------
# Training side (Alg. 2 and the backward-pass equations of Section 4.2)
# --------------------------------------------------------------------------
def couple(W: np.ndarray, g, h):
    """Alg. 2, forward loop, with the scales given: R_0 = W; for i = 1..K:
    B_i = sign(R_{i-1}); W_hat_i = g_i (.) B_i (.) h_i; R_i = R_{i-1} - W_hat_i.

    The sign of a residual decides a stored bit, so the precision of the
    residual is part of the definition: fp32 (the shared weight of a training
    step), one rounding for the product g_i[r] * h_i[c] and one for the
    subtraction (B_i only flips the sign of the product, which is exact).
    g [K][out], h [K][in] are widened exactly to fp32.
    Returns (signs int8 [K][out][in], R_K float32 [out][in])."""
    R = np.array(W, dtype=np.float32, copy=True)
    g32 = np.asarray(g).astype(np.float32)
    h32 = np.asarray(h).astype(np.float32)
    K = g32.shape[0]
    signs = np.empty((K,) + R.shape, dtype=np.int8)
    for i in range(K):
        B = sign(R)
        prod = (g32[i][:, None] * h32[i][None, :]).astype(np.float32)
        R = (R - np.where(B > 0, prod, -prod)).astype(np.float32)
        signs[i] = B
    return signs, R


def weight_grad(Delta, X) -> np.ndarray:
    """Eq. (RaBiT-grad-wfp): dL/dW_hat = (dL/dY) X^T with X [in][N], Y [out][N];
    here tokens are rows: Delta [N][out], X [N][in] -> [out][in], fp64."""
    return _f64(Delta).T @ _f64(X)


def scale_grads(signs: np.ndarray, g, h, X, Delta):
    """Eq. (RaBiT-grad-gh), binary cores held constant:
        grad g_i = sum_n Delta_n (.) (B_i (h_i (.) x_n))
        grad h_i = sum_n (B_i^T (Delta_n (.) g_i)) (.) x_n
    X [N][in], Delta [N][out]; returns (grad_g [K][out], grad_h [K][in]), fp64,
    written sample by sample as the equation is."""
    B = np.asarray(signs).astype(np.float64)
    g = _f64(g)
    h = _f64(h)
    X = _f64(X)
    D = _f64(Delta)
    K = B.shape[0]
    gg = np.zeros_like(g)
    gh = np.zeros_like(h)
    for n in range(X.shape[0]):
        for i in range(K):
            gg[i] += D[n] * (B[i] @ (h[i] * X[n]))
            gh[i] += (B[i].T @ (D[n] * g[i])) * X[n]
    return gg, gh


# --------------------------------------------------------------------------
# Stack of layers
# --------------------------------------------------------------------------
def stack_forward(layers: Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray]],
                  ops: Sequence[Tuple[int, int, int]],
                  bufs: List[Optional[np.ndarray]],
                  forced_inputs: Optional[Sequence[np.ndarray]] = None) -> List[np.ndarray]:
    """Run ops (layer, src, dst) in order.  ``bufs[src]`` holds fp16 [T][in].

    Free-running mode (``forced_inputs`` None): every op's fp64 output is
    rounded to fp16 (round-to-nearest-even) and stored in ``bufs[dst]`` for the
    ops that read it.  Teacher-forced mode: op n reads ``forced_inputs[n]``
    instead (the input another implementation actually saw), so rounding
    differences do not compound.  Returns each op's fp64 output [T][out].
    """
    outs = []
    for n, (layer, src, dst) in enumerate(ops):
        signs, g, h = layers[layer]
        x = bufs[src] if forced_inputs is None else forced_inputs[n]
        y = forward(signs, g, h, x)
        outs.append(y)
        if forced_inputs is None:
            bufs[dst] = y.astype(np.float16)
    return outs


# --------------------------------------------------------------------------
# The decoder block around the layers (Section 5.4: Llama-2 decoding)
# --------------------------------------------------------------------------
EPI_NONE, EPI_ADD, EPI_SILU_MUL = 0, 1, 2


def rmsnorm(X, w, eps: float) -> np.ndarray:
    """x / sqrt(mean_j x_j^2 + eps) (.) w for every row of X [T][n]; fp64."""
    X = _f64(X)
    X = X.reshape(-1, X.shape[-1])
    w = _f64(w).reshape(-1)
    ms = (X * X).sum(axis=1, keepdims=True) / X.shape[1]
    return X / np.sqrt(ms + eps) * w[None, :]


def silu(z) -> np.ndarray:
    """z * sigmoid(z) = z / (1 + exp(-z)); fp64."""
    z = _f64(z)
    with np.errstate(over="ignore"):
        return z / (1.0 + np.exp(-z))


def block_forward(layers: Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray]],
                  norm_weights: Sequence[np.ndarray], eps: float,
                  ops: Sequence[Tuple[int, int, int, int, int, int]],
                  bufs: List[Optional[np.ndarray]], write_back: bool = True) -> List[np.ndarray]:
    """Run ops (layer, src, dst, norm, epilogue, aux) in order; returns each op's fp64 output.

    The layer's input is ``bufs[src]`` (fp16 [T][in]), normalised with
    ``norm_weights[norm]`` first when ``norm >= 0``.  Epilogues on the layer's
    output y: EPI_NONE: y;  EPI_ADD: y + bufs[aux] (the residual stream);
    EPI_SILU_MUL: silu(y) * y_up, where y_up is layer ``aux`` applied to the
    same input (the gate and up projections of the feed-forward part).
    With ``write_back`` the result, rounded to fp16, becomes ``bufs[dst]``
    (free-running); without it ``bufs`` is only read, so a caller can hand in
    the buffers another implementation produced (teacher-forced).
    """
    outs = []
    for layer, src, dst, norm, epilogue, aux in ops:
        x = _f64(bufs[src])
        x = x.reshape(-1, x.shape[-1])
        if norm >= 0:
            x = rmsnorm(x, norm_weights[norm], eps)
        signs, g, h = layers[layer]
        y = forward(signs, g, h, x)
        if epilogue == EPI_ADD:
            y = y + _f64(bufs[aux]).reshape(y.shape)
        elif epilogue == EPI_SILU_MUL:
            signs_u, g_u, h_u = layers[aux]
            y = silu(y) * forward(signs_u, g_u, h_u, x)
        elif epilogue != EPI_NONE:
            raise ValueError("unknown epilogue")
        outs.append(y)
        if write_back:
            bufs[dst] = y.astype(np.float16)
    return outs
