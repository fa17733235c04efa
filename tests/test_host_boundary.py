"""CPU-only checks of the C-ABI library: it loads, exports what the header
declares, packs bit-exactly like the oracle, and turns bad arguments into
status codes (no compute call runs here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import synth
import paper_2602_05367_amd as rb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "rabit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rb_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    declared = _declared_functions()
    assert "rb_pack" in declared and "rb_linear_gemv" in declared and "rb_layer_stack" in declared
    for name in declared:
        assert hasattr(rb.lib, name), name
    assert sorted(rb.EXPORTS) == declared


@pytest.mark.parametrize("shape", [(1, 1, 32), (2, 16, 256), (2, 37, 160), (1, 50, 544), (2, 64, 1024), (3, 21, 288)])
def test_pack_is_bit_exact_against_oracle(shape):
    rng = synth.child_rng(0, 100, *shape)
    signs = synth.uniform_signs(rng, *shape)
    packed = rb.rb_pack(signs)
    assert packed.dtype == np.uint32
    assert np.array_equal(packed, oracle.pack(signs))
    assert np.array_equal(rb.rb_unpack(packed), signs)
    assert np.array_equal(rb.rb_unpack(oracle.pack(signs)), oracle.unpack(packed))


@pytest.mark.parametrize("shape", [(1, 1, 32), (2, 16, 256), (2, 37, 160), (1, 50, 544), (2, 33, 1056), (3, 18, 544)])
def test_native_layout_round_trip_and_size(shape):
    K, out, inn = shape
    rng = synth.child_rng(0, 101, *shape)
    packed = oracle.pack(synth.uniform_signs(rng, K, out, inn))
    native = rb.rb_repack_native(packed)
    rt, ct = -(-out // 16), -(-inn // 256)
    assert native.nbytes == rb.rb_native_bytes(K, out, inn) == rt * ct * 64 * 2 * K * 4
    assert np.array_equal(rb.rb_unpack_native(native, K, out, inn), packed)
    # same multiset of bits apart from zero padding
    assert int(np.bitwise_count(native).sum()) == int(np.bitwise_count(packed).sum())


def test_native_layout_places_words_as_documented():
    K, out, inn = 2, 32, 512
    packed = np.arange(K * out * (inn // 32), dtype=np.uint32).reshape(K, out, inn // 32) + 1
    native = rb.rb_repack_native(packed).reshape(2, 2, 64, 2, K)   # [rt][ct][lane][c][k]
    for rt, ct, lane, c, k in [(0, 0, 0, 0, 0), (1, 1, 63, 1, 1), (0, 1, 17, 1, 0), (1, 0, 40, 0, 1)]:
        row, q = rt * 16 + lane % 16, lane // 16
        canonical = int(packed[k, row, ct * 8 + c * 4 + q])
        word = int(native[rt, ct, lane, c, k])
        for e in range(8):
            for s in range(4):                       # native bit 4e+s is column 8s+e of the word
                assert (word >> (4 * e + s)) & 1 == (canonical >> (8 * s + e)) & 1


def test_pack_error_codes():
    i8 = np.ones((1, 2, 32), dtype=np.int8)
    out = np.zeros(2, dtype=np.uint32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert rb.lib.rb_pack(None, 1, 2, 32, p(out)) == rb.RB_ERR_NULL
    assert rb.lib.rb_pack(p(i8), 1, 2, 32, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_pack(p(i8), 1, 2, 48, p(out)) == rb.RB_ERR_SHAPE
    assert rb.lib.rb_pack(p(i8), 0, 2, 32, p(out)) == rb.RB_ERR_SHAPE
    assert rb.lib.rb_pack(p(i8), 4, 2, 32, p(out)) == rb.RB_ERR_SHAPE
    bad = i8.copy(); bad[0, 1, 5] = 0
    assert rb.lib.rb_pack(p(bad), 1, 2, 32, p(out)) == rb.RB_ERR_VALUE
    assert rb.rb_native_bytes(2, 16, 48) == 0


def test_compute_entry_points_reject_bad_arguments_without_a_gpu():
    """Validation happens before anything is enqueued, so it can run here."""
    L = rb.binding.rb_layer(64, 256, 2, 0x1000, 0x2000, 0x3000)
    ref = ctypes.byref
    gemm = rb.lib.rb_linear_gemm
    assert gemm(None, 0x10, 0x20, 1, 0, 0, None, 0, None) == rb.RB_ERR_NULL
    assert gemm(ref(L), None, 0x20, 1, 0, 0, None, 0, None) == rb.RB_ERR_NULL
    assert gemm(ref(L), 0x10, 0x20, 0, 0, 0, None, 0, None) == rb.RB_ERR_SHAPE
    assert gemm(ref(L), 0x10, 0x24, 1, 0, 0, None, 0, None) == rb.RB_ERR_ALIGN
    assert gemm(ref(L), 0x10, 0x20, 1, 7, 0, None, 0, None) == rb.RB_ERR_UNSUPPORTED
    assert gemm(ref(L), 0x10, 0x20, 1, 0, 9, None, 0, None) == rb.RB_ERR_UNSUPPORTED
    for field, value, code in [("inn", 250, rb.RB_ERR_SHAPE), ("K", 4, rb.RB_ERR_SHAPE),
                               ("out", 0, rb.RB_ERR_SHAPE), ("bits", 0, rb.RB_ERR_NULL),
                               ("bits", 0x1004, rb.RB_ERR_ALIGN), ("g", 0, rb.RB_ERR_NULL)]:
        bad = rb.binding.rb_layer(64, 256, 2, 0x1000, 0x2000, 0x3000)
        setattr(bad, field, value)
        assert gemm(ref(bad), 0x10, 0x20, 1, 0, 0, None, 0, None) == code, field
        assert rb.lib.rb_linear_gemv(ref(bad), 0x10, 0x20, None, 0, None) == code, field
    ops = (rb.binding.rb_stack_op * 1)(rb.binding.rb_stack_op(0, 0, 0))
    bufs = (ctypes.c_void_p * 2)(0x100, 0x200)
    stack = rb.lib.rb_layer_stack
    assert stack(ref(L), 1, ops, 1, bufs, 2, 1, None, 0, None) == rb.RB_ERR_SHAPE      # src == dst
    ops[0] = rb.binding.rb_stack_op(1, 0, 1)
    assert stack(ref(L), 1, ops, 1, bufs, 2, 1, None, 0, None) == rb.RB_ERR_SHAPE      # layer index
    ops[0] = rb.binding.rb_stack_op(0, 0, 2)
    assert stack(ref(L), 1, ops, 1, bufs, 2, 1, None, 0, None) == rb.RB_ERR_SHAPE      # buffer index
    assert stack(None, 1, ops, 1, bufs, 2, 1, None, 0, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_dense_gemv_f16(0x10, 0x20, 0x30, 4, 12, None) == rb.RB_ERR_SHAPE
    assert rb.lib.rb_stream_read(0x10, 24, 0x20, None) == rb.RB_ERR_SHAPE


def test_block_entry_points_reject_bad_arguments_without_a_gpu():
    B = rb.binding.rb_block_op
    ref = ctypes.byref
    layers = (rb.binding.rb_layer * 2)(rb.binding.rb_layer(64, 256, 2, 0x1000, 0x2000, 0x3000),
                                       rb.binding.rb_layer(32, 256, 2, 0x1000, 0x2000, 0x3000))
    bufs = (ctypes.c_void_p * 3)(0x100, 0x200, 0x300)
    norms = (ctypes.c_void_p * 1)(0x400)
    prep = rb.lib.rb_block_prepare

    def call(op, n_norms=1, eps=1e-5, T=1):
        ops = (B * 1)(op)
        return prep(layers, 2, norms, n_norms, eps, ops, 1, bufs, 3, T, 0x10000, 1 << 40, None)
    assert call(B(0, 0, 0, -1, rb.RB_EPI_NONE, -1)) == rb.RB_ERR_SHAPE            # src == dst
    assert call(B(0, 0, 1, 1, rb.RB_EPI_NONE, -1)) == rb.RB_ERR_SHAPE             # norm index
    assert call(B(0, 0, 1, 0, rb.RB_EPI_NONE, -1), n_norms=0) == rb.RB_ERR_SHAPE
    assert call(B(0, 0, 1, -1, 7, -1)) == rb.RB_ERR_SHAPE                         # unknown epilogue
    assert call(B(0, 0, 1, -1, rb.RB_EPI_ADD, 3)) == rb.RB_ERR_SHAPE              # buffer index of the addend
    assert call(B(0, 0, 1, -1, rb.RB_EPI_ADD, 0)) == rb.RB_ERR_SHAPE              # adding the op's own input
    assert call(B(0, 0, 1, -1, rb.RB_EPI_SILU_MUL, 2)) == rb.RB_ERR_SHAPE         # layer index of up
    assert call(B(0, 0, 1, -1, rb.RB_EPI_SILU_MUL, 1)) == rb.RB_ERR_SHAPE         # gate and up differ in shape
    assert call(B(0, 0, 1, -1, rb.RB_EPI_NONE, -1), eps=-1.0) == rb.RB_ERR_SHAPE
    assert call(B(0, 0, 1, -1, rb.RB_EPI_NONE, -1), T=0) == rb.RB_ERR_SHAPE
    ops = (B * 1)(B(0, 0, 1, -1, rb.RB_EPI_NONE, -1))
    assert prep(layers, 2, norms, 1, 1e-5, ops, 1, bufs, 3, 1, 0x10000, 16, None) == rb.RB_ERR_WORKSPACE
    assert prep(None, 2, norms, 1, 1e-5, ops, 1, bufs, 3, 1, 0x10000, 1 << 40, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_block_workspace_bytes(layers, 2, 1, 1) > rb.lib.rb_workspace_bytes(layers, 2, 1, 1)
    assert rb.lib.rb_rmsnorm(None, 0x10, 0x20, 1, 8, 1e-5, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_rmsnorm(0x10, 0x10, 0x20, 0, 8, 1e-5, None) == rb.RB_ERR_SHAPE
    assert rb.lib.rb_silu_mul(0x10, None, 0x20, 8, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_add(0x10, 0x10, 0x20, 0, None) == rb.RB_ERR_SHAPE


def test_derivation_entry_point_rejects_bad_arguments_without_a_gpu():
    d = rb.lib.rb_derive_iterative
    ok = dict(W=0x1000, rf=None, cf=None, K=2, T=3, out=16, inn=64, packed=0x2000, g=0x3000, h=0x4000, err=None,
              ws=0x10000, n=1 << 30)

    def call(**kw):
        a = dict(ok, **kw)
        return d(a["W"], a["rf"], a["cf"], a["K"], a["T"], a["out"], a["inn"], a["packed"], a["g"], a["h"], a["err"],
                 a["ws"], a["n"], None)
    assert call(W=None) == rb.RB_ERR_NULL and call(g=None) == rb.RB_ERR_NULL
    assert call(K=0) == rb.RB_ERR_SHAPE and call(K=4) == rb.RB_ERR_SHAPE and call(T=0) == rb.RB_ERR_SHAPE
    assert call(inn=40) == rb.RB_ERR_SHAPE and call(out=0) == rb.RB_ERR_SHAPE
    assert call(g=0x3004) == rb.RB_ERR_ALIGN and call(packed=0x2002) == rb.RB_ERR_ALIGN
    assert call(n=64) == rb.RB_ERR_WORKSPACE and call(ws=None) == rb.RB_ERR_WORKSPACE
    assert rb.lib.rb_derive_workspace_bytes(16, 40) == 0
    assert rb.lib.rb_derive_workspace_bytes(4096, 4096) > 4096 * 4096 // 8


def test_storage_accounting_reproduces_effective_bits():
    """K*out*in/8 sign bytes + fp16 scales: ~2.02 bits per weight at 4096x4096
    (Section 4.1) and ~2.01 over the whole 7B-shaped stack."""
    ops, _ = synth.llama_stack("7b")
    sign_bytes = sum(2 * op.out * op.inn // 8 for op in ops)
    assert sign_bytes == 1_619_001_344
    scale_bytes = sum(2 * 2 * (op.out + op.inn) for op in ops)
    weights = sum(op.out * op.inn for op in ops)
    assert round(8 * (sign_bytes + scale_bytes) / weights, 2) == 2.01
    assert round(8 * (2 * 4096 * 4096 // 8 + 2 * 2 * 8192) / 4096 ** 2, 2) == 2.02
    ops13, _ = synth.llama_stack("13b")
    assert sum(2 * op.out * op.inn // 8 for op in ops13) == 3_171_942_400
    # the native layout adds no bytes when out % 16 == 0 and in % 256 == 0
    assert rb.rb_native_bytes(2, 4096, 11008) == 2 * 4096 * 11008 // 8


def test_many_token_workspace_counts_the_shared_last_round():
    """The many-token GEMM needs 256 bytes for the power-of-two scalings, 256 bytes per 32-column
    group for the input scales in operand order, the input in fp16 in contraction order (T x in)
    and, when the output tiles (256 rows x 256 tokens) do not fill whole rounds of the device's 256
    compute units, fp32 partial sums for the row blocks of the last round, one copy per workgroup
    that shares a tile."""
    def need(out, inn, T):
        L = rb.binding.rb_layer(out, inn, 2, 0x1000, 0x2000, 0x3000)
        return rb.lib.rb_workspace_bytes(ctypes.byref(L), 1, 1, T)
    T = 2048
    u = lambda inn: 256 + (inn // 32) * 256 + T * inn * 2
    # 112 x 8 = 896 tiles = 3.5 rounds: the last 16 row blocks (4096 rows), two workgroups per tile
    assert need(28672, 8192, T) == u(8192) + 2 * T * 4096 * 4
    # 32 x 8 = 256 tiles: one full round, nothing shared
    assert need(8192, 28672, T) == u(28672)
    # 16 x 8 = 128 tiles: half a round, every tile shared by two
    assert need(4096, 4096, T) == u(4096) + 2 * T * 4096 * 4
    # 43 x 8 = 344 tiles: one round, then 88 tiles (rows 8192..11007) shared by two
    assert need(11008, 4096, T) == u(4096) + 2 * T * (11008 - 8192) * 4
