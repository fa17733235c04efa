"""ctypes binding of librabit.so: argument marshalling only.

Every function has the name and meaning of the C entry point in
``include/rabit.h``.  PyTorch supplies device memory and the current stream;
all arithmetic runs in the HIP kernels.  Importing this module fails loudly if
the library has not been built - there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Sequence, Tuple

import numpy as np
import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librabit.so")

RB_OK = 0
RB_ERR_NULL, RB_ERR_SHAPE, RB_ERR_ALIGN, RB_ERR_UNSUPPORTED = -1, -2, -3, -4
RB_ERR_HIP, RB_ERR_WORKSPACE, RB_ERR_VALUE, RB_ERR_HANDOVER = -5, -6, -7, -8
RB_F16, RB_BF16, RB_F32 = 0, 1, 2
_ERR_NAMES = {-1: "RB_ERR_NULL", -2: "RB_ERR_SHAPE", -3: "RB_ERR_ALIGN", -4: "RB_ERR_UNSUPPORTED",
              -5: "RB_ERR_HIP", -6: "RB_ERR_WORKSPACE", -7: "RB_ERR_VALUE", -8: "RB_ERR_HANDOVER"}

EXPORTS = [
    "rb_pack", "rb_unpack", "rb_native_bytes", "rb_repack_native", "rb_unpack_native",
    "rb_linear_gemv", "rb_linear_gemm", "rb_layer_stack", "rb_workspace_bytes",
    "rb_stack_prepare", "rb_stack_run", "rb_stack_forget", "rb_stack_status", "rb_stack_waited",
    "rb_stack_set_option", "rb_stack_gave_up",
    "rb_linear_gemm_noalloc", "rb_noalloc_scratch_bytes",
    "rb_couple", "rb_weight_grad", "rb_scale_grads", "rb_scale_grads_workspace_bytes",
    "rb_block_prepare", "rb_block_workspace_bytes", "rb_rmsnorm", "rb_silu_mul", "rb_add",
    "rb_derive_iterative", "rb_derive_workspace_bytes",
    "rb_dense_gemv_f16", "rb_stream_read", "rb_stream_read_groups", "rb_version", "rb_last_path",
]


class RabitError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} returned {_ERR_NAMES.get(code, code)}")
        self.code = code


class rb_layer(ctypes.Structure):
    _fields_ = [("out", ctypes.c_int), ("inn", ctypes.c_int), ("K", ctypes.c_int),
                ("bits", ctypes.c_void_p), ("g", ctypes.c_void_p), ("h", ctypes.c_void_p)]


class rb_stack_op(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_int), ("src", ctypes.c_int), ("dst", ctypes.c_int)]


class rb_block_op(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_int), ("src", ctypes.c_int), ("dst", ctypes.c_int),
                ("norm", ctypes.c_int), ("epilogue", ctypes.c_int), ("aux", ctypes.c_int)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(LIB_PATH)
    i, p, z = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.rb_pack.argtypes = [p, i, i, i, p]
    lib.rb_unpack.argtypes = [p, i, i, i, p]
    lib.rb_native_bytes.argtypes = [i, i, i]
    lib.rb_native_bytes.restype = z
    lib.rb_repack_native.argtypes = [p, i, i, i, p]
    lib.rb_unpack_native.argtypes = [p, i, i, i, p]
    lib.rb_linear_gemv.argtypes = [ctypes.POINTER(rb_layer), p, p, p, z, p]
    lib.rb_linear_gemm.argtypes = [ctypes.POINTER(rb_layer), p, p, i, i, i, p, z, p]
    lib.rb_linear_gemm_noalloc.argtypes = [ctypes.POINTER(rb_layer), p, p, i, i, i, p]
    lib.rb_noalloc_scratch_bytes.argtypes = []
    lib.rb_noalloc_scratch_bytes.restype = z
    lib.rb_layer_stack.argtypes = [ctypes.POINTER(rb_layer), i, ctypes.POINTER(rb_stack_op), i,
                                   ctypes.POINTER(ctypes.c_void_p), i, i, p, z, p]
    lib.rb_stack_prepare.argtypes = lib.rb_layer_stack.argtypes
    lib.rb_stack_run.argtypes = [p, z, p]
    lib.rb_stack_forget.argtypes = [p]
    lib.rb_stack_set_option.argtypes = [i, i]
    lib.rb_stack_status.argtypes = [p, p]
    lib.rb_stack_waited.argtypes = [p, p, ctypes.POINTER(ctypes.c_ulonglong)]
    lib.rb_stack_gave_up.argtypes = [p, p, ctypes.POINTER(ctypes.c_int)]
    lib.rb_workspace_bytes.argtypes = [ctypes.POINTER(rb_layer), i, i, i]
    lib.rb_workspace_bytes.restype = z
    lib.rb_block_workspace_bytes.argtypes = [ctypes.POINTER(rb_layer), i, i, i]
    lib.rb_block_workspace_bytes.restype = z
    lib.rb_block_prepare.argtypes = [ctypes.POINTER(rb_layer), i, ctypes.POINTER(ctypes.c_void_p), i, ctypes.c_float,
                                     ctypes.POINTER(rb_block_op), i, ctypes.POINTER(ctypes.c_void_p), i, i, p, z, p]
    lib.rb_rmsnorm.argtypes = [p, p, p, i, i, ctypes.c_float, p]
    lib.rb_silu_mul.argtypes = [p, p, p, z, p]
    lib.rb_add.argtypes = [p, p, p, z, p]
    lib.rb_derive_workspace_bytes.argtypes = [i, i]
    lib.rb_derive_workspace_bytes.restype = z
    lib.rb_derive_iterative.argtypes = [p, p, p, i, i, i, i, p, p, p, p, p, z, p]
    lib.rb_couple.argtypes = [p, p, p, i, i, i, p, p, p, p]
    lib.rb_weight_grad.argtypes = [p, p, i, i, i, p, p]
    lib.rb_scale_grads_workspace_bytes.argtypes = [i, i, i]
    lib.rb_scale_grads_workspace_bytes.restype = z
    lib.rb_scale_grads.argtypes = [p, p, p, p, i, i, i, p, p, p, z, p]
    lib.rb_dense_gemv_f16.argtypes = [p, p, p, i, i, p]
    lib.rb_stream_read.argtypes = [p, z, p, p]
    lib.rb_stream_read_groups.argtypes = []
    lib.rb_version.argtypes = []
    lib.rb_last_path.argtypes = []
    for name in EXPORTS:
        if name not in ("rb_native_bytes", "rb_workspace_bytes", "rb_noalloc_scratch_bytes",
                        "rb_scale_grads_workspace_bytes", "rb_block_workspace_bytes", "rb_derive_workspace_bytes"):
            getattr(lib, name).restype = i
    return lib


lib = _load()


def _check(fn: str, code: int) -> None:
    if code != RB_OK:
        raise RabitError(fn, code)


def _np_ptr(a: np.ndarray) -> ctypes.c_void_p:
    return a.ctypes.data_as(ctypes.c_void_p)


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_DTYPE_CODE = {torch.float16: RB_F16, torch.bfloat16: RB_BF16, torch.float32: RB_F32}


# ------------------------------------------------------------------ host ---
def rb_pack(signs: np.ndarray) -> np.ndarray:
    """int8 +1/-1 [K][out][in] (host) -> canonical uint32 [K][out][in/32] (host)."""
    signs = np.ascontiguousarray(signs, dtype=np.int8)
    K, out, inn = signs.shape
    packed = np.empty((K, out, max(inn // 32, 0)), dtype=np.uint32)
    _check("rb_pack", lib.rb_pack(_np_ptr(signs), K, out, inn, _np_ptr(packed)))
    return packed


def rb_unpack(packed: np.ndarray) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    K, out, W32 = packed.shape
    signs = np.empty((K, out, W32 * 32), dtype=np.int8)
    _check("rb_unpack", lib.rb_unpack(_np_ptr(packed), K, out, W32 * 32, _np_ptr(signs)))
    return signs


def rb_native_bytes(K: int, out: int, inn: int) -> int:
    return int(lib.rb_native_bytes(K, out, inn))


def rb_repack_native(packed: np.ndarray) -> np.ndarray:
    """canonical uint32 [K][out][in/32] -> native layout, flat uint32 (host)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    K, out, W32 = packed.shape
    native = np.empty(rb_native_bytes(K, out, W32 * 32) // 4, dtype=np.uint32)
    _check("rb_repack_native", lib.rb_repack_native(_np_ptr(packed), K, out, W32 * 32, _np_ptr(native)))
    return native


def rb_unpack_native(native: np.ndarray, K: int, out: int, inn: int) -> np.ndarray:
    native = np.ascontiguousarray(native, dtype=np.uint32)
    packed = np.empty((K, out, inn // 32), dtype=np.uint32)
    _check("rb_unpack_native", lib.rb_unpack_native(_np_ptr(native), K, out, inn, _np_ptr(packed)))
    return packed


# ---------------------------------------------------------------- device ---
class Layer:
    """Device-resident frozen layer: native sign words + fp16 g [K][out], h [K][in]."""

    def __init__(self, bits: torch.Tensor, g: torch.Tensor, h: torch.Tensor, K: int, out: int, inn: int):
        assert bits.is_cuda and g.is_cuda and h.is_cuda
        assert g.dtype == torch.float16 and h.dtype == torch.float16
        assert tuple(g.shape) == (K, out) and tuple(h.shape) == (K, inn)
        assert bits.numel() * bits.element_size() == rb_native_bytes(K, out, inn)
        self.bits, self.g, self.h = bits.contiguous(), g.contiguous(), h.contiguous()
        self.K, self.out, self.inn = K, out, inn

    @classmethod
    def from_host(cls, signs: np.ndarray, g: np.ndarray, h: np.ndarray, device="cuda:0") -> "Layer":
        """Pack int8 signs [K][out][in] with rb_pack + rb_repack_native and upload."""
        K, out, inn = signs.shape
        native = rb_repack_native(rb_pack(signs))
        bits = torch.from_numpy(native.view(np.int32)).to(device)
        return cls(bits, torch.from_numpy(np.ascontiguousarray(g, dtype=np.float16)).to(device),
                   torch.from_numpy(np.ascontiguousarray(h, dtype=np.float16)).to(device), K, out, inn)

    def struct(self) -> rb_layer:
        return rb_layer(self.out, self.inn, self.K, self.bits.data_ptr(), self.g.data_ptr(),
                        self.h.data_ptr())

    @property
    def packed_bytes(self) -> int:
        """Bytes of sign bits of the unpadded matrix (K*out*in/8)."""
        return self.K * self.out * self.inn // 8


def _layer_array(layers: Sequence[Layer]):
    arr = (rb_layer * len(layers))()
    for n, L in enumerate(layers):
        arr[n] = L.struct()
    return arr


def rb_workspace_bytes(layers: Sequence[Layer], n_ops: int, T: int) -> int:
    return int(lib.rb_workspace_bytes(_layer_array(layers), len(layers), n_ops, T))


def _workspace(layers: Sequence[Layer], T: int, device, n_ops: int = 1) -> Tuple[torch.Tensor, int]:
    n = rb_workspace_bytes(layers, n_ops, T)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=device)
    return ws, n


def rb_linear_gemv(layer: Layer, x: torch.Tensor, y: torch.Tensor = None, workspace=None) -> torch.Tensor:
    """y = layer(x) for one fp16 token x [in]; returns fp16 [out]."""
    assert x.is_cuda and x.dtype == torch.float16 and x.is_contiguous() and x.numel() == layer.inn
    if y is None:
        y = torch.empty(layer.out, dtype=torch.float16, device=x.device)
    ws, n = workspace if workspace is not None else _workspace([layer], 1, x.device)
    s = layer.struct()
    _check("rb_linear_gemv", lib.rb_linear_gemv(ctypes.byref(s), x.data_ptr(), y.data_ptr(),
                                                ws.data_ptr(), n, _stream()))
    return y


def rb_linear_gemm(layer: Layer, X: torch.Tensor, out_dtype=torch.float16, Y: torch.Tensor = None,
                   workspace=None) -> torch.Tensor:
    """Y[t] = layer(X[t]); X [T][in] fp16 or bf16; returns [T][out] of out_dtype."""
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.inn
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, layer.out), dtype=out_dtype, device=X.device)
    ws, n = workspace if workspace is not None else _workspace([layer], T, X.device)
    s = layer.struct()
    _check("rb_linear_gemm", lib.rb_linear_gemm(ctypes.byref(s), X.data_ptr(), Y.data_ptr(), T,
                                                _DTYPE_CODE[X.dtype], _DTYPE_CODE[Y.dtype],
                                                ws.data_ptr(), n, _stream()))
    return Y


def rb_linear_gemm_noalloc(layer: Layer, X: torch.Tensor, Y: torch.Tensor) -> torch.Tensor:
    """rb_linear_gemm_noalloc: like rb_linear_gemm, scratch memory inside the library; the caller
    passes the output tensor, so that nothing is allocated on the way."""
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.inn
    assert Y.is_cuda and Y.is_contiguous() and tuple(Y.shape) == (X.shape[0], layer.out)
    s = layer.struct()
    _check("rb_linear_gemm_noalloc", lib.rb_linear_gemm_noalloc(
        ctypes.byref(s), X.data_ptr(), Y.data_ptr(), X.shape[0], _DTYPE_CODE[X.dtype], _DTYPE_CODE[Y.dtype],
        _stream()))
    return Y


def rb_noalloc_scratch_bytes() -> int:
    return int(lib.rb_noalloc_scratch_bytes())


class Stack:
    """Marshalled arguments of rb_layer_stack, built once and reused per call."""

    def __init__(self, layers: Sequence[Layer], ops: Sequence[Tuple[int, int, int]],
                 bufs: Sequence[torch.Tensor], T: int):
        self.layers, self.bufs, self.T = list(layers), list(bufs), T
        for b in self.bufs:
            assert b.is_cuda and b.dtype == torch.float16 and b.is_contiguous()
        self._layers = _layer_array(self.layers)
        self._ops = (rb_stack_op * len(ops))(*[rb_stack_op(*o) for o in ops])
        self._bufs = (ctypes.c_void_p * len(bufs))(*[b.data_ptr() for b in self.bufs])
        self.n_ops = len(ops)
        self.ws, self.ws_bytes = _workspace(self.layers, T, self.bufs[0].device, n_ops=len(ops))

    def run(self) -> None:
        """rb_layer_stack: set-up and execution in one call."""
        _check("rb_layer_stack", lib.rb_layer_stack(
            self._layers, len(self.layers), self._ops, self.n_ops, self._bufs, len(self.bufs), self.T,
            self.ws.data_ptr(), self.ws_bytes, _stream()))

    def prepare(self) -> None:
        """rb_stack_prepare: everything that does not depend on the activations."""
        _check("rb_stack_prepare", lib.rb_stack_prepare(
            self._layers, len(self.layers), self._ops, self.n_ops, self._bufs, len(self.bufs), self.T,
            self.ws.data_ptr(), self.ws_bytes, _stream()))

    def run_prepared(self) -> None:
        """rb_stack_run: one pass of the prepared ops over the current buffer contents."""
        _check("rb_stack_run", lib.rb_stack_run(self.ws.data_ptr(), self.ws_bytes, _stream()))

    def status(self) -> int:
        """rb_stack_status: waits for the stream; RB_OK, or RB_ERR_HANDOVER if a run gave up a wait."""
        return int(lib.rb_stack_status(self.ws.data_ptr(), _stream()))

    def waited(self) -> int:
        """rb_stack_waited: input tiles, over all runs since prepare, that were requested before they
        were written and had to be waited for (waits for the stream)."""
        n = ctypes.c_ulonglong(0)
        _check("rb_stack_waited", lib.rb_stack_waited(self.ws.data_ptr(), _stream(), ctypes.byref(n)))
        return int(n.value)

    def gave_up(self) -> int:
        """rb_stack_gave_up: which bounded wait a run gave up (0: none); waits for the stream."""
        r = ctypes.c_int(0)
        _check("rb_stack_gave_up", lib.rb_stack_gave_up(self.ws.data_ptr(), _stream(), ctypes.byref(r)))
        return int(r.value)

    def forget(self) -> None:
        _check("rb_stack_forget", lib.rb_stack_forget(self.ws.data_ptr()))


RB_EPI_NONE, RB_EPI_ADD, RB_EPI_SILU_MUL = 0, 1, 2


class Block(Stack):
    """Marshalled arguments of rb_block_prepare; run, status, waited and forget are the stack's."""

    def __init__(self, layers: Sequence[Layer], norm_weights: Sequence[torch.Tensor], eps: float,
                 ops: Sequence[Tuple[int, int, int, int, int, int]], bufs: Sequence[torch.Tensor], T: int):
        self.layers, self.bufs, self.T = list(layers), list(bufs), T
        self.norm_weights, self.eps = list(norm_weights), float(eps)
        for b in self.bufs + self.norm_weights:
            assert b.is_cuda and b.dtype == torch.float16 and b.is_contiguous()
        self._layers = _layer_array(self.layers)
        self._ops = (rb_block_op * len(ops))(*[rb_block_op(*o) for o in ops])
        self._bufs = (ctypes.c_void_p * len(bufs))(*[b.data_ptr() for b in self.bufs])
        self._norms = (ctypes.c_void_p * max(len(self.norm_weights), 1))(*[w.data_ptr() for w in self.norm_weights])
        self.n_ops = len(ops)
        self.ws_bytes = int(lib.rb_block_workspace_bytes(self._layers, len(self.layers), self.n_ops, T))
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device=self.bufs[0].device)

    def run(self) -> None:
        self.prepare()
        self.run_prepared()

    def prepare(self) -> None:
        """rb_block_prepare: everything that does not depend on the activations."""
        _check("rb_block_prepare", lib.rb_block_prepare(
            self._layers, len(self.layers), self._norms, len(self.norm_weights), self.eps, self._ops, self.n_ops,
            self._bufs, len(self.bufs), self.T, self.ws.data_ptr(), self.ws_bytes, _stream()))


def rb_rmsnorm(x: torch.Tensor, w: torch.Tensor, eps: float, y: torch.Tensor = None) -> torch.Tensor:
    """y[t] = x[t] / sqrt(mean(x[t]^2) + eps) * w for fp16 x [T][n]."""
    assert x.is_cuda and x.dtype == torch.float16 and x.is_contiguous() and x.dim() == 2
    assert w.dtype == torch.float16 and w.numel() == x.shape[1]
    if y is None:
        y = torch.empty_like(x)
    _check("rb_rmsnorm", lib.rb_rmsnorm(x.data_ptr(), w.data_ptr(), y.data_ptr(), x.shape[0], x.shape[1], float(eps),
                                        _stream()))
    return y


def rb_silu_mul(gate: torch.Tensor, up: torch.Tensor, y: torch.Tensor = None) -> torch.Tensor:
    assert gate.is_cuda and gate.dtype == torch.float16 and up.dtype == torch.float16
    assert gate.is_contiguous() and up.is_contiguous() and gate.shape == up.shape
    if y is None:
        y = torch.empty_like(gate)
    _check("rb_silu_mul", lib.rb_silu_mul(gate.data_ptr(), up.data_ptr(), y.data_ptr(), gate.numel(), _stream()))
    return y


def rb_add(a: torch.Tensor, b: torch.Tensor, y: torch.Tensor = None) -> torch.Tensor:
    assert a.is_cuda and a.dtype == torch.float16 and b.dtype == torch.float16
    assert a.is_contiguous() and b.is_contiguous() and a.shape == b.shape
    if y is None:
        y = torch.empty_like(a)
    _check("rb_add", lib.rb_add(a.data_ptr(), b.data_ptr(), y.data_ptr(), a.numel(), _stream()))
    return y


def rb_layer_stack(layers: Sequence[Layer], ops: Sequence[Tuple[int, int, int]],
                   bufs: Sequence[torch.Tensor], T: int) -> None:
    """Run ops (layer, src, dst) in order over device fp16 buffers [T][width]."""
    Stack(layers, ops, bufs, T).run()


def rb_dense_gemv_f16(W: torch.Tensor, x: torch.Tensor, y: torch.Tensor = None) -> torch.Tensor:
    out, inn = W.shape
    assert W.dtype == torch.float16 and x.dtype == torch.float16 and W.is_contiguous()
    if y is None:
        y = torch.empty(out, dtype=torch.float16, device=W.device)
    _check("rb_dense_gemv_f16", lib.rb_dense_gemv_f16(W.data_ptr(), x.data_ptr(), y.data_ptr(), out, inn,
                                                      _stream()))
    return y


def rb_stream_read(src: torch.Tensor, sink: torch.Tensor = None) -> torch.Tensor:
    nbytes = src.numel() * src.element_size()
    if sink is None:
        sink = torch.empty(int(lib.rb_stream_read_groups()) * 16, dtype=torch.uint8, device=src.device)
    _check("rb_stream_read", lib.rb_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream()))
    return sink


RB_PATH_NONE, RB_PATH_SIGNADD, RB_PATH_MX, RB_PATH_GEMM, RB_PATH_BATCH = 0, 1, 2, 3, 4
RB_OPT_HANDOVER_PAUSE = 1


# -------------------------------------------------------- initialisation ---
def rb_derive_iterative(W: torch.Tensor, K: int, T_max: int, row_factors: torch.Tensor = None,
                        col_factors: torch.Tensor = None, want_err: bool = True):
    """Alg. 1 on the device: returns (packed int32 [K][out][in/32], g fp64 [K][out], h fp64 [K][in],
    err fp64 [T_max][K] or None)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.dim() == 2
    out, inn = W.shape
    for f, n in ((row_factors, out), (col_factors, inn)):
        assert f is None or (f.is_cuda and f.dtype == torch.float64 and f.is_contiguous() and f.numel() == n)
    packed = torch.empty((K, out, inn // 32), dtype=torch.int32, device=W.device)
    g = torch.empty((K, out), dtype=torch.float64, device=W.device)
    h = torch.empty((K, inn), dtype=torch.float64, device=W.device)
    err = torch.empty((T_max, K), dtype=torch.float64, device=W.device) if want_err else None
    n = int(lib.rb_derive_workspace_bytes(out, inn))
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=W.device)
    _check("rb_derive_iterative", lib.rb_derive_iterative(
        W.data_ptr(), row_factors.data_ptr() if row_factors is not None else None,
        col_factors.data_ptr() if col_factors is not None else None, K, T_max, out, inn,
        packed.data_ptr(), g.data_ptr(), h.data_ptr(), err.data_ptr() if err is not None else None,
        ws.data_ptr(), n, _stream()))
    return packed, g, h, err


# -------------------------------------------------------------- training ---
def rb_couple(W: torch.Tensor, g: torch.Tensor, h: torch.Tensor, want_native: bool = True,
              want_residual: bool = False):
    """Alg. 2 forward loop on the device: W fp32 [out][in], g fp16 [K][out], h fp16 [K][in] ->
    (packed uint32 [K][out][in/32] as int32 tensor, native flat int32 tensor or None, residual or None)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous()
    assert g.dtype == torch.float16 and h.dtype == torch.float16 and g.is_contiguous() and h.is_contiguous()
    out, inn = W.shape
    K = g.shape[0]
    packed = torch.empty((K, out, inn // 32), dtype=torch.int32, device=W.device)
    native = torch.empty(rb_native_bytes(K, out, inn) // 4, dtype=torch.int32, device=W.device) if want_native else None
    residual = torch.empty_like(W) if want_residual else None
    _check("rb_couple", lib.rb_couple(W.data_ptr(), g.data_ptr(), h.data_ptr(), K, out, inn, packed.data_ptr(),
                                      native.data_ptr() if native is not None else None,
                                      residual.data_ptr() if residual is not None else None, _stream()))
    return packed, native, residual


def rb_weight_grad(Delta: torch.Tensor, X: torch.Tensor) -> torch.Tensor:
    """G = Delta^T X in fp32: Delta fp16 [N][out], X fp16 [N][in]."""
    assert Delta.is_cuda and Delta.dtype == torch.float16 and X.dtype == torch.float16
    assert Delta.is_contiguous() and X.is_contiguous() and Delta.shape[0] == X.shape[0]
    N, out = Delta.shape
    inn = X.shape[1]
    G = torch.empty((out, inn), dtype=torch.float32, device=X.device)
    _check("rb_weight_grad", lib.rb_weight_grad(Delta.data_ptr(), X.data_ptr(), N, out, inn, G.data_ptr(), _stream()))
    return G


def rb_scale_grads(G: torch.Tensor, packed: torch.Tensor, g: torch.Tensor, h: torch.Tensor):
    """(grad_g fp32 [K][out], grad_h fp32 [K][in]) from G fp32 [out][in] and the canonical packed cores."""
    assert G.is_cuda and G.dtype == torch.float32 and G.is_contiguous() and packed.is_contiguous()
    out, inn = G.shape
    K = g.shape[0]
    n = int(lib.rb_scale_grads_workspace_bytes(K, out, inn))
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=G.device)
    gg = torch.empty((K, out), dtype=torch.float32, device=G.device)
    gh = torch.empty((K, inn), dtype=torch.float32, device=G.device)
    _check("rb_scale_grads", lib.rb_scale_grads(G.data_ptr(), packed.data_ptr(), g.data_ptr(), h.data_ptr(), K, out, inn,
                                                gg.data_ptr(), gh.data_ptr(), ws.data_ptr(), n, _stream()))
    return gg, gh


def rb_stack_set_option(option: int, value: int) -> None:
    _check("rb_stack_set_option", lib.rb_stack_set_option(option, value))


def rb_last_path() -> int:
    return int(lib.rb_last_path())


def rb_version() -> int:
    return int(lib.rb_version())
