"""Many-token matrix-core GEMM vs the fp64 oracle (Section 4.1, Eq. stacked binary
weight), through the C ABI.  Sizes span several 256 x 256 workgroup tiles and ragged
tails in every dimension; the 70B-shaped prefill matrices are checked on sampled
outputs the oracle computes one by one."""
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


@pytest.mark.parametrize("out,inn,T", [
    (256, 256, 256),        # exactly one workgroup tile, one column tile
    (512, 1024, 300),       # two row blocks, ragged tokens
    (272, 320, 33),         # ragged rows (17 row tiles), ragged columns (in % 256 != 0)
    (1000, 2080, 517),      # everything ragged, three token blocks
    (48, 32, 3),            # tiny: one row tile group, the smallest input width
    (4096, 1024, 256),      # 16 output tiles on 256 compute units: every tile's contraction cut in four
    (8400, 1024, 2048),     # 264 tiles: one full round, then 8 tiles (ragged last row block) cut in four
    (2816, 512, 2048),      # 88 tiles: cut in two, as many slices as column tiles
])
def test_gemm_matches_oracle(out, inn, T):
    rng = synth.child_rng(5, 100, out, inn, T)
    signs, g, h = random_layer(rng, 2, out, inn)
    X = synth.outlier_activations(rng, T, inn)
    _say(f"gemm out={out} in={inn} T={T}")
    L = to_device_layer(signs, g, h)
    Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_GEMM
    err = max_rel_l2(Y, oracle.forward(signs, g, h, X))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL


@pytest.mark.parametrize("out,inn,T", [(272, 320, 33), (1000, 2080, 517), (4096, 1024, 256), (8400, 1024, 300)])
def test_three_path_gemm_matches_oracle(out, inn, T):
    """The 3-bit variant beyond 32 tokens: the same one-contraction kernel with a third path in
    the effective weight (ragged shapes, tiles cut along the contraction, scales of either sign)."""
    rng = synth.child_rng(5, 110, out, inn, T)
    signs, g, h = random_layer(rng, 3, out, inn)
    g = g.copy(); h = h.copy()
    g[2, ::7] *= -1; h[1, ::5] *= -1; h[2, 3::4] *= -1; g[0, 11] = 0
    X = synth.outlier_activations(rng, T, inn)
    _say(f"three-path gemm out={out} in={inn} T={T}")
    L = to_device_layer(signs, g, h)
    Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_GEMM
    err = max_rel_l2(Y, oracle.forward(signs, g, h, X))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL


@pytest.mark.parametrize("out,inn,T,bf16_in,path", [
    (272, 544, 5, False, "generic"), (272, 544, 6, False, "batch"), (1000, 2080, 8, False, "batch"), (272, 544, 12, False, "batch"),
    (272, 544, 13, False, "gemm"), (1000, 2080, 32, False, "gemm"), (272, 544, 3, True, "generic"), (48, 32, 7, True, "gemm")])
def test_three_path_single_calls_at_few_tokens(out, inn, T, bf16_in, path):
    """One call on a three-path layer at 6..32 tokens reads the weights once: the small-batch kernel
    as a plan of one op up to 12 fp16 tokens, the one-contraction kernel beyond that and for bf16."""
    rng = synth.child_rng(5, 111, out, inn, T)
    signs, g, h = random_layer(rng, 3, out, inn)
    g = g.copy(); h = h.copy()
    g[1, ::6] *= -1; h[2, ::3] *= -1
    X = synth.outlier_activations(rng, T, inn)
    _say(f"three-path single call out={out} in={inn} T={T} bf16={bf16_in}")
    L = to_device_layer(signs, g, h)
    Xd = torch.from_numpy(X).cuda()
    if bf16_in:
        Xd = Xd.to(torch.bfloat16)
        X = oracle.bf16_bits_to_f64(bf16_bits(Xd.cpu())).reshape(T, inn)
    Y = rb.rb_linear_gemm(L, Xd)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == {"batch": rb.RB_PATH_BATCH, "gemm": rb.RB_PATH_GEMM, "generic": rb.RB_PATH_SIGNADD}[path]
    err = max_rel_l2(Y, oracle.forward(signs, g, h, X))
    _say(f"  rel_l2={err:.3e}")
    assert err <= TOL


def test_gemm_negative_and_zero_scales():
    """Stored output scales of either sign and zero: the kernel folds the sign of g into the
    sign bits and keeps |g| as the magnitude of its left operand."""
    out, inn, T = 96, 512, 40
    rng = synth.child_rng(5, 101)
    signs, g, h = random_layer(rng, 2, out, inn)
    g = g.copy(); h = h.copy()
    g[0, ::3] *= -1; g[1, 1::4] *= -1; g[1, 5] = 0
    h[0, ::5] *= -1; h[1, 7] = 0
    X = synth.gaussian_activations(rng, T, inn)
    L = to_device_layer(signs, g, h)
    Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_GEMM
    assert max_rel_l2(Y, oracle.forward(signs, g, h, X)) <= TOL


@pytest.mark.parametrize("T", [16, 70])
def test_gemm_when_the_magnitude_sits_in_g(T):
    """Section 4.1 leaves the split of a path's magnitude between g and h open.  With h around 3e-5
    and g around 10 the products h x are fp16 subnormals unless the kernel scales each path's h by
    a power of two first (and takes it back out of g); path 2 gets another factor 1/8 on h."""
    out, inn = 272, 1056
    rng = synth.child_rng(5, 109, T)
    signs, g, h = random_layer(rng, 2, out, inn)
    g = (g.astype(np.float64) * 500.0 * np.array([1.0, 8.0])[:, None]).astype(np.float16)
    h = (h.astype(np.float64) * 2.0e-3 * np.array([1.0, 1.0 / 8.0])[:, None]).astype(np.float16)
    assert np.all(np.isfinite(g.astype(np.float64))) and np.count_nonzero(h) > 0.9 * h.size
    X = synth.outlier_activations(rng, T, inn)
    L = to_device_layer(signs, g, h)
    Y = rb.rb_linear_gemm(L, torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_GEMM
    assert max_rel_l2(Y, oracle.forward(signs, g, h, X)) <= TOL


def test_gemm_rows_equal_single_token_calls():
    out, inn, T = 320, 1536, 70
    rng = synth.child_rng(5, 102)
    signs, g, h = random_layer(rng, 2, out, inn)
    X = synth.gaussian_activations(rng, T, inn)
    L = to_device_layer(signs, g, h)
    Xd = torch.from_numpy(X).cuda()
    Y = rb.rb_linear_gemm(L, Xd).cpu().numpy().astype(np.float64)
    for t in (0, 31, T - 1):
        yt = rb.rb_linear_gemv(L, Xd[t].contiguous())
        assert max_rel_l2(yt, Y[t][None]) <= 2e-3


@pytest.mark.parametrize("out,inn", [(28672, 8192), (8192, 28672)])
def test_prefill_70b_shapes_sampled(out, inn):
    """Config 5 at full size (T = 2048, bf16 activations, uniform signs drawn on the device in
    native order): 64 sampled outputs per call, each computed by the oracle from the unpacked
    row, plus two whole token rows of a 512-row slice."""
    T = 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(20260205 + out)
    nbytes = rb.rb_native_bytes(2, out, inn)
    bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda", generator=gen)
    rng = synth.child_rng(5, 103, out)
    g = synth.halfnormal_scales(rng, 2, out); h = synth.halfnormal_scales(rng, 2, inn)
    g[1] *= np.float16(0.3); h[1] *= np.float16(0.3)
    L = rb.Layer(bits, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), 2, out, inn)
    Xt = torch.randn((T, inn), device="cuda", generator=gen).to(torch.bfloat16)
    _say(f"prefill {out}x{inn} T={T}")
    Y = rb.rb_linear_gemm(L, Xt, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_GEMM
    # unpack the sampled rows on the host with the library's own (bit-exact, CPU-tested) unpacker
    native = bits.cpu().numpy().view(np.uint32)
    packed = rb.rb_unpack_native(native, 2, out, inn)
    signs_rows = lambda rows: rb.rb_unpack(packed[:, rows, :])
    pick = np.random.default_rng(7)
    rows = np.unique(pick.integers(0, out, size=64)); toks = pick.integers(0, T, size=len(rows))
    S = signs_rows(rows)                                            # [2][n][in]
    X64 = oracle.bf16_bits_to_f64(bf16_bits(Xt[torch.from_numpy(toks).cuda()].cpu())).reshape(len(rows), inn)
    ref = np.array([oracle.forward(S[:, i:i + 1, :], g[:, rows[i]:rows[i] + 1], h, X64[i:i + 1])[0, 0]
                    for i in range(len(rows))])
    got = Y[torch.from_numpy(toks).cuda(), torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    scale = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(got - ref)) <= 4 * TOL * scale, (np.max(np.abs(got - ref)), scale)
    # two whole token rows over a 512-row slice: per-vector relative L2 as everywhere else
    # (for 28672 rows also the last 512: the row blocks of the partly filled last round, whose
    # contraction is shared by two workgroups)
    for r0 in ([3 * 512, out - 512] if out >= 2048 * 2 else [0]):
        rows2 = np.arange(r0, r0 + 512)
        S2 = signs_rows(rows2)
        for t in (0, T - 1):
            x64 = oracle.bf16_bits_to_f64(bf16_bits(Xt[t:t + 1].cpu())).reshape(1, inn)
            ref2 = oracle.forward(S2, g[:, rows2], h, x64)
            err = max_rel_l2(Y[t:t + 1, r0:r0 + 512], ref2)
            _say(f"  rows {r0}.. t={t} rel_l2={err:.3e}")
            assert err <= TOL
