"""Alg. 1 on the device (rb_derive_iterative) against the oracle's derive_iterative: both sides
decide the signs in fp64, so the stored bits must agree; scales and errors agree to what the
different summation orders leave."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb

pytestmark = pytest.mark.gpu


def _factors(rng, out, inn, alpha_in, alpha_out):
    s_in = np.abs(rng.standard_normal(inn)) + 0.1
    s_out = np.abs(rng.standard_normal(out)) + 0.1
    rows = (s_out / s_out.max()) ** alpha_out
    cols = (s_in / s_in.max()) ** alpha_in
    return s_in, s_out, rows, cols


def _run(W, K, T_max, rows=None, cols=None):
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).cuda()
    packed, g, h, err = rb.rb_derive_iterative(torch.from_numpy(W).cuda(), K, T_max, dev(rows), dev(cols))
    torch.cuda.synchronize()
    return packed.cpu().numpy().view(np.uint32), g.cpu().numpy(), h.cpu().numpy(), err.cpu().numpy()


@pytest.mark.parametrize("K,out,inn,T_max,calibrated", [
    (1, 7, 32, 2, False), (2, 37, 96, 4, True), (3, 130, 544, 3, True), (2, 300, 1056, 3, False), (2, 1024, 2048, 2, True)])
def test_iterative_svid_matches_the_oracle(K, out, inn, T_max, calibrated):
    rng = synth.child_rng(7, 700, K, out)
    W = synth.gaussian_weight(rng, out, inn, std=0.02).astype(np.float32)
    W[0, :3] = 0.0
    print(f"derive K={K} {out}x{inn} T_max={T_max} calibrated={calibrated}", flush=True)
    if calibrated:
        s_in, s_out, rows, cols = _factors(rng, out, inn, 0.5, 0.25)
        signs, g, h, err = oracle.derive_iterative(W, K, T_max, s_in=s_in, s_out=s_out, alpha_in=0.5, alpha_out=0.25)
        got = _run(W, K, T_max, rows, cols)
    else:
        signs, g, h, err = oracle.derive_iterative(W, K, T_max)
        got = _run(W, K, T_max)
    packed, g_d, h_d, err_d = got
    ref_packed = oracle.pack(signs)
    differing = int(np.unpackbits((packed ^ ref_packed).view(np.uint8)).sum())
    assert differing == 0, f"{differing} of {signs.size} signs differ"
    np.testing.assert_allclose(g_d, g, rtol=1e-8, atol=1e-14)
    np.testing.assert_allclose(h_d, h, rtol=1e-8, atol=1e-14)
    np.testing.assert_allclose(err_d, err, rtol=1e-9)
    # and what the method promises: every update lowers the error
    flat = err_d.reshape(-1)
    assert np.all(np.diff(flat) <= 1e-12 * flat[0])


def test_one_sweep_is_the_greedy_pass():
    """T_max = 1 against the oracle's greedy derivation, a function of its own."""
    rng = synth.child_rng(7, 701)
    W = synth.gaussian_weight(rng, 272, 544, std=0.02).astype(np.float32)
    signs, g, h, norms = oracle.derive(W, 3, round_scales=False)
    packed, g_d, h_d, err_d = _run(W, 3, 1)
    assert np.array_equal(packed, oracle.pack(signs))
    np.testing.assert_allclose(g_d, g, rtol=1e-8)
    np.testing.assert_allclose(h_d, h, rtol=1e-8)
    np.testing.assert_allclose(err_d[0], norms[1:], rtol=1e-9)
    # residual fractions of a Gaussian weight: 1 - 2/pi, 0.130, 0.058
    frac = (norms[1:] / norms[0]) ** 2
    assert abs(frac[0] - (1 - 2 / np.pi)) < 0.01 and abs(frac[1] - 0.130) < 0.01 and abs(frac[2] - 0.058) < 0.01


def test_degenerate_weights():
    # all zero: no scale, every sign +1
    packed, g, h, err = _run(np.zeros((20, 64), dtype=np.float32), 2, 2)
    assert not packed.any() and not g.any() and not h.any() and not err.any()
    # a weight that is one path exactly: found in the first update, nothing left for the second
    rng = synth.child_rng(7, 702)
    B = synth.uniform_signs(rng, 1, 48, 96)[0].astype(np.float64)
    g0, h0 = np.abs(rng.standard_normal(48)) + 0.5, np.abs(rng.standard_normal(96)) + 0.5
    W = (g0[:, None] * B * h0[None, :]).astype(np.float32)
    packed, g, h, err = _run(W, 2, 1)
    assert np.array_equal(packed[0], oracle.pack(B[None].astype(np.int8))[0])
    np.testing.assert_allclose(g[0][:, None] * h[0][None, :], np.abs(W.astype(np.float64)), rtol=1e-6)
    assert err[0, 0] <= 1e-6 * np.linalg.norm(W) and err[0, 1] <= err[0, 0]


def test_derived_paths_run_through_the_inference_kernel():
    """Initialise on the device, round the scales to fp16, tile the signs, run a token: the
    oracle's forward on the oracle's own initialisation must agree."""
    rng = synth.child_rng(7, 703)
    out, inn, K = 528, 1056, 2
    W = synth.gaussian_weight(rng, out, inn, std=0.02).astype(np.float32)
    signs, g, h, _ = oracle.derive_iterative(W, K, 3)
    packed, g_d, h_d, _ = _run(W, K, 3)
    g16, h16 = g_d.astype(np.float16), h_d.astype(np.float16)
    assert np.array_equal(g16, g.astype(np.float16)) and np.array_equal(h16, h.astype(np.float16))
    native = torch.from_numpy(rb.rb_repack_native(packed).view(np.int32)).cuda()
    L = rb.Layer(native, torch.from_numpy(g16).cuda(), torch.from_numpy(h16).cuda(), K, out, inn)
    x = synth.gaussian_activations(rng, 1, inn)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    ref = oracle.forward(signs, g.astype(np.float16), h.astype(np.float16), x)
    assert oracle.relative_l2(y.cpu().numpy().astype(np.float64)[None], ref).max() <= 1e-3


def test_full_size_layer_as_benchmarked_last_update_against_the_oracle():
    """4096 x 11008, K = 2, the size bench.py times.  The oracle cannot run the whole iteration at
    this size in test time, but the last update of the last sweep is an SVID of one residual that
    numpy can form from what the device returned for the other path: its signs must be the stored
    bits of path 2, the oracle's leading singular pair of its magnitudes the stored scales, and the
    remaining error the last entry of the error table.  The errors must fall from update to update
    and start at the greedy values of a Gaussian weight (residual fractions 1 - 2/pi and 0.130)."""
    out, inn, K, T_max = 4096, 11008, 2, 2
    W = (torch.randn((out, inn), device="cuda", generator=torch.Generator(device="cuda").manual_seed(7)) * 0.02)
    print("derive 4096x11008 on the device", flush=True)
    packed, g, h, err = rb.rb_derive_iterative(W, K, T_max)
    torch.cuda.synchronize()
    Wh = W.cpu().numpy().astype(np.float64)
    packed, g, h, err = packed.cpu().numpy().view(np.uint32), g.cpu().numpy(), h.cpu().numpy(), err.cpu().numpy()
    norm = np.linalg.norm(Wh)
    flat = err.reshape(-1)
    assert np.all(np.diff(flat) < 0)
    assert abs((flat[0] / norm) ** 2 - (1 - 2 / np.pi)) < 0.003 and abs((flat[1] / norm) ** 2 - 0.130) < 0.003
    print("  residual of path 2 in numpy", flush=True)
    B0 = oracle.unpack(packed[0:1])[0]
    R = Wh - g[0][:, None] * B0 * h[0][None, :]
    del B0
    B1 = oracle.sign(R)
    differing = int(np.unpackbits((oracle.pack(B1[None]) ^ packed[1:2]).view(np.uint8)).sum())
    assert differing == 0, differing
    sigma, a, b = oracle.leading_singular_pair(np.abs(R))
    np.testing.assert_allclose(g[1], np.sqrt(sigma) * a, rtol=1e-8)
    np.testing.assert_allclose(h[1], np.sqrt(sigma) * b, rtol=1e-8)
    left = np.linalg.norm(R - g[1][:, None] * B1 * h[1][None, :])
    np.testing.assert_allclose(flat[-1], left, rtol=1e-9)
