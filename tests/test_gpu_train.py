"""Training-side kernels against the oracle: the coupled derivation of the binary cores (bit-exact:
the residual's precision is part of the definition) and the gradients of the scales."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb

pytestmark = pytest.mark.gpu


def _scales(rng, K, n, scale):
    return (np.abs(rng.standard_normal((K, n))) * scale * (0.6 ** np.arange(K))[:, None]).astype(np.float16)


@pytest.mark.parametrize("K,out,inn", [(1, 7, 32), (2, 37, 96), (3, 130, 544), (2, 272, 1056), (2, 1024, 4096)])
def test_couple_bits_and_residual_are_the_oracles(K, out, inn):
    rng = synth.child_rng(5, 600, K, out)
    W = synth.gaussian_weight(rng, out, inn, std=1.0).astype(np.float32)
    W[0, :5] = 0.0                                            # sign(0) = +1
    g, h = _scales(rng, K, out, 0.9), _scales(rng, K, inn, 0.9)
    signs, R = oracle.couple(W, g, h)
    print(f"couple K={K} {out}x{inn}", flush=True)
    packed, native, residual = rb.rb_couple(torch.from_numpy(W).cuda(), torch.from_numpy(g).cuda(),
                                            torch.from_numpy(h).cuda(), want_native=True, want_residual=True)
    torch.cuda.synchronize()
    ref_packed = oracle.pack(signs)
    got_packed = packed.cpu().numpy().view(np.uint32)
    assert np.array_equal(got_packed, ref_packed)
    # the native tiles are what the host repacker makes of the canonical words, padding included
    assert np.array_equal(native.cpu().numpy().view(np.uint32), rb.rb_repack_native(ref_packed))
    assert np.array_equal(residual.cpu().numpy(), R)          # same roundings, bit for bit
    # packed only, native only
    p2, n2, r2 = rb.rb_couple(torch.from_numpy(W).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(),
                              want_native=False)
    assert n2 is None and r2 is None and torch.equal(p2, packed)


def test_coupled_cores_run_through_the_inference_kernels():
    """A training step's forward pass: derive the cores on the device, feed the native tiles to the
    decode kernel, compare with the oracle's forward on the oracle's cores."""
    rng = synth.child_rng(5, 601)
    out, inn, K = 528, 1056, 2
    W = synth.gaussian_weight(rng, out, inn, std=0.02).astype(np.float32)
    _, g, h, _ = oracle.derive(W, K)
    signs, _ = oracle.couple(W, g, h)
    x = synth.gaussian_activations(rng, 1, inn)
    gd, hd = torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda()
    _, native, _ = rb.rb_couple(torch.from_numpy(W).cuda(), gd, hd)
    L = rb.Layer(native, gd, hd, K, out, inn)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    ref = oracle.forward(signs, g, h, x)
    assert oracle.relative_l2(y.cpu().numpy().astype(np.float64)[None], ref).max() <= 1e-3


@pytest.mark.parametrize("K,out,inn,N", [(1, 5, 32, 1), (2, 37, 96, 3), (3, 130, 544, 4), (2, 300, 1056, 7)])
def test_scale_gradients_against_the_oracle(K, out, inn, N):
    """fp32 sums of out or in terms against fp64: 1e-5 relative to the gradient's norm (the bound
    for recursive fp32 summation of a few thousand terms of mixed sign is ~n * 2^-24 of the sum of
    magnitudes; the measured error is an order below)."""
    rng = synth.child_rng(5, 602, K, out)
    signs = synth.uniform_signs(rng, K, out, inn)
    g, h = _scales(rng, K, out, 0.5), _scales(rng, K, inn, 0.5)
    X = synth.gaussian_activations(rng, N, inn)
    D = (rng.standard_normal((N, out)) * 0.1).astype(np.float16)
    ref_g, ref_h = oracle.scale_grads(signs, g, h, X, D)
    print(f"scale gradients K={K} {out}x{inn} N={N}", flush=True)
    G = rb.rb_weight_grad(torch.from_numpy(D).cuda(), torch.from_numpy(X).cuda())
    packed = torch.from_numpy(oracle.pack(signs).view(np.int32)).cuda()
    gg, gh = rb.rb_scale_grads(G, packed, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda())
    gg2, gh2 = rb.rb_scale_grads(G, packed, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda())
    torch.cuda.synchronize()
    assert torch.equal(gg, gg2) and torch.equal(gh, gh2)      # fixed summation order
    refG = oracle.weight_grad(D, X)
    assert np.abs(G.cpu().numpy() - refG).max() <= 1e-5 * np.abs(refG).max()
    for got, ref in ((gg, ref_g), (gh, ref_h)):
        err = np.linalg.norm(got.cpu().numpy().astype(np.float64) - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert err.max() <= 1e-5, err


def test_training_entry_points_reject_bad_arguments():
    W = torch.zeros((4, 32), dtype=torch.float32, device="cuda")
    g = torch.zeros((2, 4), dtype=torch.float16, device="cuda")
    h = torch.zeros((2, 32), dtype=torch.float16, device="cuda")
    out = torch.zeros((2, 4, 1), dtype=torch.int32, device="cuda")
    lib = rb.lib
    assert lib.rb_couple(W.data_ptr(), g.data_ptr(), h.data_ptr(), 2, 4, 32, None, None, None, None) == rb.RB_ERR_NULL
    assert lib.rb_couple(None, g.data_ptr(), h.data_ptr(), 2, 4, 32, out.data_ptr(), None, None, None) == rb.RB_ERR_NULL
    assert lib.rb_couple(W.data_ptr(), g.data_ptr(), h.data_ptr(), 4, 4, 32, out.data_ptr(), None, None, None) == rb.RB_ERR_SHAPE
    assert lib.rb_couple(W.data_ptr(), g.data_ptr(), h.data_ptr(), 2, 4, 33, out.data_ptr(), None, None, None) == rb.RB_ERR_SHAPE
    # the kernels read W sixteen and h eight bytes at a time
    assert lib.rb_couple(W.data_ptr() + 4, g.data_ptr(), h.data_ptr(), 2, 3, 32, out.data_ptr(), None, None, None) == rb.RB_ERR_ALIGN
    assert lib.rb_couple(W.data_ptr(), g.data_ptr(), h.data_ptr() + 2, 1, 4, 32, out.data_ptr(), None, None, None) == rb.RB_ERR_ALIGN
    assert lib.rb_scale_grads(W.data_ptr(), out.data_ptr(), g.data_ptr(), h.data_ptr(), 2, 4, 32, W.data_ptr(), W.data_ptr(),
                              None, 0, None) == rb.RB_ERR_WORKSPACE
    assert lib.rb_scale_grads_workspace_bytes(2, 4, 31) == 0
