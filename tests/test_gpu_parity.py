"""HIP path vs the fp64 oracle, element by element on the same seeded inputs.
Every call goes through the C ABI (ctypes binding)."""
import sys

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb
from helpers import TOL, random_layer, to_device_layer, bf16_bits, max_rel_l2

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_config1_single_layer_2048():
    out, inn, K = synth.single_layer_config()
    rng = synth.child_rng(1, 0)
    signs, g, h = random_layer(rng, K, out, inn)
    x = synth.gaussian_activations(rng, 1, inn)
    _say(f"config1 gemv out={out} in={inn} K={K}")
    L = to_device_layer(signs, g, h)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX          # K=2, one fp16 token: the matrix-core kernel
    err = max_rel_l2(y, oracle.forward(signs, g, h, x))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL


# several tiles + ragged tails: out not a multiple of 16, in not a multiple of 256
@pytest.mark.parametrize("K,out,inn", [
    (1, 1, 32), (2, 1, 32), (2, 16, 256), (2, 17, 288), (1, 50, 544), (2, 100, 1056),
    (2, 257, 4096 + 32), (1, 64, 8192), (2, 48, 4096 * 2 + 256), (2, 333, 11008 // 4),
    (3, 16, 256), (3, 100, 1056), (3, 257, 4096 + 32),
])
def test_gemv_shapes_and_tails(K, out, inn):
    rng = synth.child_rng(0, 200, K, out, inn)
    signs, g, h = random_layer(rng, K, out, inn)
    x = synth.gaussian_activations(rng, 1, inn)
    _say(f"gemv K={K} out={out} in={inn}")
    L = to_device_layer(signs, g, h)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == (rb.RB_PATH_MX if K == 2 else rb.RB_PATH_SIGNADD)
    err = max_rel_l2(y, oracle.forward(signs, g, h, x))
    _say(f"  rel_l2={err:.3e} path={rb.rb_last_path()}")
    assert err <= TOL


def test_three_paths_derived_and_batched():
    """K = 3 (the 3-bit variant of the paper's packing appendix): paths derived from a Gaussian
    matrix, one token and a few on the generic kernel, a small batch on the small-batch kernel."""
    rng = synth.child_rng(0, 260)
    W = rng.standard_normal((160, 544)) * 0.02
    signs, g, h, norms = oracle.derive(W, 3)
    assert norms[3] < norms[2] < norms[1] < norms[0]
    L = to_device_layer(signs, g, h)
    for T in (1, 4, 9):
        X = synth.outlier_activations(rng, T, 544)
        _say(f"K=3 derived 160x544 T={T}")
        Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda())
        torch.cuda.synchronize()
        assert rb.rb_last_path() == (rb.RB_PATH_SIGNADD if T <= 4 else rb.RB_PATH_BATCH)
        assert max_rel_l2(Y, oracle.forward(signs, g, h, X)) <= TOL
        # the third path refines the second: closer to the dense W x than the two-path layer
        dense = (X.astype(np.float64) @ W.T)
        e3 = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - dense)
        e2 = np.linalg.norm(oracle.forward(signs[:2], g[:2], h[:2], X) - dense)
        assert e3 < e2


def test_probe_vectors_recover_every_stored_bit():
    """x = e_j  =>  y_i = sum_k g_k[i] B_k[i][j] h_k[j]: checks the native layout
    and the kernel's indexing bit by bit (scales are powers of two, so exact)."""
    K, out, inn = 2, 40, 544
    rng = synth.child_rng(0, 201)
    signs = synth.uniform_signs(rng, K, out, inn)
    g = np.stack([np.full(out, 1.0), np.full(out, 0.25)]).astype(np.float16)
    h = np.stack([np.full(inn, 1.0), np.full(inn, 0.5)]).astype(np.float16)
    L = to_device_layer(signs, g, h)
    X = np.eye(inn, dtype=np.float16)
    _say(f"probe vectors K={K} out={out} in={inn}")
    Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda()).cpu().numpy().astype(np.float64)
    expect = (signs[0].astype(np.float64) * 1.0 + signs[1].astype(np.float64) * 0.125).T
    assert np.array_equal(Y, expect)


def test_all_plus_one_gives_plain_sum_and_single_flip():
    K, out, inn = 1, 32, 512
    rng = synth.child_rng(0, 202)
    signs = np.ones((K, out, inn), dtype=np.int8)
    ones_o = np.ones((K, out), dtype=np.float16); ones_i = np.ones((K, inn), dtype=np.float16)
    x = (rng.integers(-8, 9, size=(1, inn)) / 8.0).astype(np.float16)       # exact arithmetic
    L = to_device_layer(signs, ones_o, ones_i)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda()).cpu().numpy().astype(np.float64)
    assert np.all(y == x.astype(np.float64).sum())
    signs[0, 7, 300] = -1
    L2 = to_device_layer(signs, ones_o, ones_i)
    y2 = rb.rb_linear_gemv(L2, torch.from_numpy(x[0]).cuda()).cpu().numpy().astype(np.float64)
    d = y2 - y
    assert d[7] == -2.0 * float(x[0, 300]) and np.all(np.delete(d, 7) == 0)


@pytest.mark.parametrize("T", [2, 4, 8, 16, 5])
def test_skinny_gemm_with_outlier_channels(T):
    K, out, inn = 2, 528, 4096
    rng = synth.child_rng(3, T)
    signs, g, h = random_layer(rng, K, out, inn)
    X = synth.outlier_activations(rng, T, inn)
    _say(f"skinny gemm T={T} out={out} in={inn}")
    L = to_device_layer(signs, g, h)
    Xd = torch.from_numpy(X).cuda()
    Y = rb.rb_linear_gemm(L, Xd)
    torch.cuda.synchronize()
    err = max_rel_l2(Y, oracle.forward(signs, g, h, X))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL
    # row t of the batched call equals the single-token call
    for t in (0, T - 1):
        yt = rb.rb_linear_gemv(L, Xd[t].contiguous())
        assert max_rel_l2(yt, Y[t].cpu().numpy().astype(np.float64)[None]) <= 2e-3


@pytest.mark.parametrize("out_dtype", [torch.float16, torch.float32, torch.bfloat16])
def test_gemm_bf16_activations_and_output_types(out_dtype):
    K, out, inn, T = 2, 272, 1024, 48
    rng = synth.child_rng(5, 0)
    signs, g, h = random_layer(rng, K, out, inn)
    Xt = torch.from_numpy(rng.standard_normal((T, inn)).astype(np.float32)).to(torch.bfloat16)
    X64 = oracle.bf16_bits_to_f64(bf16_bits(Xt)).reshape(T, inn)
    L = to_device_layer(signs, g, h)
    _say(f"gemm bf16 in, {out_dtype} out, T={T}")
    Y = rb.rb_linear_gemm(L, Xt.cuda(), out_dtype=out_dtype)
    torch.cuda.synchronize()
    err = max_rel_l2(Y, oracle.forward(signs, g, h, X64))
    _say(f"  rel_l2={err:.3e}")
    # a bf16 result carries 8 significant bits: its own rounding alone is ~1.7e-3 RMS
    assert err <= (TOL if out_dtype != torch.bfloat16 else 3e-3)


def test_linearity():
    K, out, inn = 2, 64, 1024
    rng = synth.child_rng(0, 203)
    signs, g, h = random_layer(rng, K, out, inn, gain=50.0)
    a = synth.gaussian_activations(rng, 1, inn)[0]; b = synth.gaussian_activations(rng, 1, inn)[0]
    L = to_device_layer(signs, g, h)
    f = lambda v: rb.rb_linear_gemv(L, torch.from_numpy(v).cuda()).cpu().numpy().astype(np.float64)
    comb = (2.0 * a.astype(np.float32) + b.astype(np.float32)).astype(np.float16)
    lhs = f(comb)
    rhs = oracle.forward(signs, g, h, comb[None])[0]
    assert oracle.relative_l2(lhs[None], rhs[None])[0] <= TOL
    assert oracle.relative_l2(lhs[None], (2.0 * f(a) + f(b))[None])[0] <= 4e-3


def test_derived_weights_from_gaussian_matrix():
    """Paths derived as the paper defines (sign, rank-1 scale fit, binarised
    residual) from W ~ N(0, 0.02^2), on a 7B-shaped slice: 4096 inputs."""
    out, inn = 512, 4096
    rng = synth.child_rng(2, 0)
    W = synth.gaussian_weight(rng, out, inn)
    signs, g, h, norms = oracle.derive(W, 2)
    x = synth.gaussian_activations(rng, 1, inn)
    L = to_device_layer(signs, g, h)
    _say("derived weights 512x4096")
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    err = max_rel_l2(y, oracle.forward(signs, g, h, x))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL
    # and the two paths together approximate the dense product (residual energy ~0.13)
    dense = x.astype(np.float64) @ W.T
    assert oracle.relative_l2(y.cpu().numpy()[None], dense)[0] < 0.5
