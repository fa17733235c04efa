"""The small-batch kernel (one pass over the weights for up to 16 tokens, two or three paths) and
the three-path form of the fused decode kernel (one token) against the oracle: every op of a stack
recomputed from the input the GPU run actually used."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb
from helpers import TOL, to_device_layer, random_layer

pytestmark = pytest.mark.gpu


def _branching_stack(rng, K, widths):
    """x -> a; a -> b, c, d (three readers of one output); b -> e; c -> f (e, f, d: stack outputs).
    widths: (x, a, b, c, d, e, f).  Gains keep activations near RMS 1 through the chain."""
    x, a, b, c, d, e, f = widths
    shapes = [(a, x), (b, a), (c, a), (d, a), (e, b), (f, c)]
    layers = []
    for (o, i) in shapes:
        signs, g, h = random_layer(rng, K, o, i)
        # half-normal scales: E[g h] ~ (0.02 * 0.8)^2 per path; bring the output to RMS ~1
        gain = 1.0 / (np.sqrt(i * K) * (0.02 * 0.02))
        layers.append((signs, (g.astype(np.float64) * gain).astype(np.float16), h))
    op_list = [(0, 0, 1), (1, 1, 2), (2, 1, 3), (3, 1, 4), (4, 2, 5), (5, 3, 6)]
    return layers, op_list


def _check_stack(layers, op_list, widths, x, T, label, prepared):
    # one token and three paths in every layer: the fused decode kernel; everything else here: the small-batch kernel
    want_path = rb.RB_PATH_MX if (T == 1 and all(l[0].shape[0] == 3 for l in layers)) else rb.RB_PATH_BATCH
    dev_layers = [to_device_layer(*l) for l in layers]
    bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    bufs[0].copy_(torch.from_numpy(x))
    print(f"{label}: T={T}, prepared={prepared}", flush=True)
    runs = []
    if prepared:
        stack = rb.Stack(dev_layers, op_list, bufs, T)
        stack.prepare()
        for _ in range(2):                      # the second run must repeat the first bit for bit
            stack.run_prepared()
            torch.cuda.synchronize()
            runs.append([b.clone() for b in bufs])
        assert rb.rb_last_path() == want_path
        assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
        stack.forget()
        for a, b in zip(*runs):
            assert torch.equal(a, b)
    else:
        rb.rb_layer_stack(dev_layers, op_list, bufs, T)
        torch.cuda.synchronize()
        assert rb.rb_last_path() == want_path
    got = [b.cpu().numpy() for b in bufs]
    worst = 0.0
    for n, (l, s, d) in enumerate(op_list):
        assert np.all(np.isfinite(got[d])), n
        ref = oracle.forward(*layers[l], got[s])
        assert np.abs(ref).max() > 0.05, n            # not a comparison of zeros
        err = float(oracle.relative_l2(got[d].astype(np.float64), ref).max())
        worst = max(worst, err)
        assert err <= TOL, (label, n, err)
    print(f"  worst rel_l2={worst:.3e}", flush=True)


# widths: part-filled row blocks (544 = 34 row tiles, 288 = 18), row counts that are not multiples of
# 16 (300, 90), column counts that are not multiples of 256 (1056, 544, 800), several column tiles
WIDTHS = (1056, 544, 288, 800, 300, 90, 1056)


@pytest.mark.parametrize("T", [5, 6, 8, 9, 13, 16])
def test_two_path_stack_small_batches(T):
    rng = synth.child_rng(3, 500, T)
    layers, op_list = _branching_stack(rng, 2, WIDTHS)
    x = synth.outlier_activations(rng, T, WIDTHS[0])
    # prepared stacks take this kernel from 8 tokens on, rb_layer_stack from 5 on
    _check_stack(layers, op_list, WIDTHS, x, T, "two paths, branching stack", prepared=(T >= 8 and T % 2 == 0))


@pytest.mark.parametrize("T", [1, 2, 4, 7, 16])
def test_three_path_stack_one_to_sixteen_tokens(T):
    rng = synth.child_rng(3, 501, T)
    layers, op_list = _branching_stack(rng, 3, WIDTHS)
    x = synth.outlier_activations(rng, T, WIDTHS[0])
    _check_stack(layers, op_list, WIDTHS, x, T, "three paths, branching stack", prepared=(T % 2 == 1))


def test_three_path_stack_derived_weights():
    """Paths derived from a Gaussian weight by the oracle (Section 4.2 steps 1-3), three paths."""
    rng = synth.child_rng(3, 502)
    shapes = [(544, 576), (288, 544), (576, 288)]
    layers = []
    x = synth.gaussian_activations(rng, 5, 576)
    cur = x
    for (o, i) in shapes:
        signs, g, h, _ = oracle.derive(synth.gaussian_weight(rng, o, i), 3)
        y = oracle.forward(signs, g, h, cur)
        g = (g.astype(np.float64) / np.sqrt((y ** 2).mean())).astype(np.float16)
        layers.append((signs, g, h))
        cur = oracle.forward(signs, g, h, cur).astype(np.float16)
    _check_stack(layers, [(0, 0, 1), (1, 1, 2), (2, 2, 3)], (576, 544, 288, 576), x, 5, "three paths, derived", True)


def test_mixed_two_and_three_path_layers_in_one_stack():
    rng = synth.child_rng(3, 503)
    shapes = [(544, 288, 2), (288, 544, 3), (320, 544, 2), (90, 288, 3)]
    layers = []
    for (o, i, K) in shapes:
        signs, g, h = random_layer(rng, K, o, i)
        gain = 1.0 / (np.sqrt(i * K) * (0.02 * 0.02))
        layers.append((signs, (g.astype(np.float64) * gain).astype(np.float16), h))
    x = synth.gaussian_activations(rng, 6, 288)          # a three-path layer: the batch kernel at any T
    # op 0: x -> a; ops 1 (K=3) and 2 (K=2) both read a; op 3 reads op 1's output
    _check_stack(layers, [(0, 0, 1), (1, 1, 2), (2, 1, 3), (3, 2, 4)], (288, 544, 288, 320, 90), x, 6, "mixed K", True)


def test_batch_kernel_with_degenerate_scales_and_extreme_inputs():
    """Negative and zero entries in g and h, an all-zero h_k, inputs at the ends of the fp16 range."""
    rng = synth.child_rng(3, 504)
    T, d0, d1, d2 = 9, 1056, 544, 270
    def edge(out, inn, zero_path):
        signs, g, h = random_layer(rng, 2, out, inn)
        g = g.astype(np.float64); h = h.astype(np.float64)
        g[:, rng.integers(0, out, 9)] *= -1.0
        h[:, rng.integers(0, inn, 17)] *= -1.0
        g[0, rng.integers(0, out, 5)] = 0.0
        h[1, rng.integers(0, inn, 11)] = 0.0
        if zero_path is not None:
            h[zero_path] = 0.0
        return signs, g.astype(np.float16), h.astype(np.float16)
    l1 = edge(d1, d0, None)
    x = synth.outlier_activations(rng, T, d0).astype(np.float64)
    idx = rng.choice(d0, size=8, replace=False)
    x[:, idx[0:2]] = 2000.0
    x[:, idx[2:4]] = 3.0e-7                                   # subnormal in fp16
    x[:, idx[4:8]] = 0.0
    x = x.astype(np.float16)
    y1 = oracle.forward(*l1, x)
    l1 = (l1[0], (l1[1].astype(np.float64) / np.sqrt((y1 ** 2).mean())).astype(np.float16), l1[2])
    l2 = edge(d2, d1, 1)
    y2 = oracle.forward(*l2, oracle.forward(*l1, x).astype(np.float16))
    l2 = (l2[0], (l2[1].astype(np.float64) / np.sqrt((y2 ** 2).mean())).astype(np.float16), l2[2])
    _check_stack([l1, l2], [(0, 0, 1), (1, 1, 2)], (d0, d1, d2), x, T, "edge cases", True)


@pytest.mark.parametrize("T,K", [(8, 2), (16, 2), (1, 3), (8, 3)])
def test_full_width_7b_block_on_the_batch_kernel(T, K):
    """One block of the 7B shape exactly as bench.py builds it (signs drawn on the device), at the
    widths and launch shapes that are timed, two and three paths: sampled rows of every op
    against the oracle."""
    import bench
    ops, layers, bufs, op_list, _ = bench.build_stack(rb, synth, torch, "7b", T, K=K)
    ops, layers, op_list = ops[:7], layers[:7], op_list[:7]
    bufs[0].copy_(torch.from_numpy(synth.outlier_activations(synth.child_rng(3, 505, T), T, ops[0].inn)))
    stack = rb.Stack(layers, op_list, bufs, T)
    stack.prepare()
    print(f"full-width 7B block on the batch kernel, T={T}, K={K}", flush=True)
    stack.run_prepared()
    torch.cuda.synchronize()
    assert rb.rb_last_path() == (rb.RB_PATH_MX if (K == 3 and T == 1) else rb.RB_PATH_BATCH) and stack.status() == rb.RB_OK
    stack.forget()
    pick = np.random.default_rng(11)
    worst = 0.0
    for n, op in enumerate(ops):
        L = layers[n]
        y = bufs[op.dst].cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(y)) and np.any(y != 0), op.name
        native = L.bits.cpu().numpy().view(np.uint32)
        packed = rb.rb_unpack_native(native, K, L.out, L.inn)
        rows = np.unique(np.concatenate([pick.integers(0, L.out, size=40), [0, L.out - 1]]))
        S = rb.rb_unpack(packed[:, rows, :])
        ref = oracle.forward(S, L.g.cpu().numpy()[:, rows], L.h.cpu().numpy(), bufs[op.src].cpu().numpy())
        err = float(oracle.relative_l2(y[:, rows], ref).max())
        worst = max(worst, err)
        assert err <= TOL, (op.name, err)
    print(f"  worst sampled rel_l2={worst:.3e}", flush=True)


@pytest.mark.parametrize("n_ops,T", [(8, 16), (4, 9), (8, 5)])
def test_many_independent_rows_take_larger_row_blocks(n_ops, T):
    """A launch with rows enough lets a workgroup own 16 (eight ops of 8192 rows) or 8 (four such
    ops) row tiles instead of 4, so that the staged inputs are shared by more rows: the same
    results, other instantiations of the kernel.  Every op reads the one stack input."""
    rng = synth.child_rng(3, 506, n_ops, T)
    out, inn = 8192 - 16 * 5 - 3, 288                 # part-filled last row tile and last row block
    layers = []
    for _ in range(n_ops):
        signs, g, h = random_layer(rng, 2, out, inn)
        gain = 1.0 / (np.sqrt(inn * 2) * (0.02 * 0.02))
        layers.append((signs, (g.astype(np.float64) * gain).astype(np.float16), h))
    x = synth.outlier_activations(rng, T, inn)
    op_list = [(n, 0, 1 + n) for n in range(n_ops)]
    _check_stack(layers, op_list, (inn,) + (out,) * n_ops, x, T, f"{n_ops} independent ops of {out} rows", prepared=(T >= 8))


@pytest.mark.parametrize("T", [1, 3, 8])
def test_scales_that_are_only_two_byte_aligned(T):
    """g and h need no more than the alignment of their elements: a two-op chain whose scale
    vectors start two bytes past a 16-byte boundary, on the fused kernel (1 and 3 tokens) and on
    the small-batch kernel (8 tokens; its input expansion reads h sixteen bytes at a time when it can)."""
    rng = synth.child_rng(3, 507, T)
    shapes = [(320, 544), (288, 320)]
    layers = [random_layer(rng, 2, o, i, gain=30.0) for o, i in shapes]

    def off_by_one(a):
        flat = torch.zeros(a.size + 1, dtype=torch.float16, device="cuda")
        flat[1:].copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float16)).flatten())
        t = flat[1:].view(a.shape)
        assert t.data_ptr() % 16 == 2
        return t
    dev_layers = []
    for signs, g, h in layers:
        aligned = to_device_layer(signs, g, h)
        dev_layers.append(rb.Layer(aligned.bits, off_by_one(g), off_by_one(h), 2, signs.shape[1], signs.shape[2]))
    x = synth.outlier_activations(rng, T, 544)
    bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in (544, 320, 288)]
    bufs[0].copy_(torch.from_numpy(x))
    print(f"scales two bytes past a 16-byte boundary, T={T}", flush=True)
    rb.rb_layer_stack(dev_layers, [(0, 0, 1), (1, 1, 2)], bufs, T)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == (rb.RB_PATH_BATCH if T == 8 else rb.RB_PATH_MX)
    got = [b.cpu().numpy() for b in bufs]
    for n, (signs, g, h) in enumerate(layers):
        ref = oracle.forward(signs, g, h, got[n])
        assert np.abs(ref).max() > 0.05
        assert oracle.relative_l2(got[n + 1].astype(np.float64), ref).max() <= TOL, n
    y = rb.rb_linear_gemm(dev_layers[0], bufs[0])             # the single-call kernels take the same layers
    torch.cuda.synchronize()
    assert oracle.relative_l2(y.cpu().numpy().astype(np.float64), oracle.forward(*layers[0], got[0])).max() <= TOL


@pytest.mark.parametrize("prepared", [True, False])
def test_three_path_decode_kernel_one_token(prepared):
    """Three paths, one token: the fused decode kernel (its three paths take the place of two
    tokens' two paths in the right operand), a branching stack with ragged widths."""
    rng = synth.child_rng(3, 507, int(prepared))
    layers, op_list = _branching_stack(rng, 3, WIDTHS)
    x = synth.outlier_activations(rng, 1, WIDTHS[0])
    _check_stack(layers, op_list, WIDTHS, x, 1, "three paths, one token", prepared)


def test_three_path_decode_kernel_early_reads_and_degenerate_scales():
    """The same kernel with no hand-over pause at all (nearly every input tile is asked for before
    it is written and has to be read again), negative and zero scales, an all-zero third path."""
    rng = synth.child_rng(3, 508)
    widths = (1056, 544, 288, 800)
    layers = []
    for n, (o, i) in enumerate([(544, 1056), (288, 544), (800, 288)]):
        signs, g, h = random_layer(rng, 3, o, i)
        g = g.astype(np.float64) / (np.sqrt(i * 3) * (0.02 * 0.02)); h = h.astype(np.float64)
        g[:, rng.integers(0, o, 7)] *= -1.0
        h[:, rng.integers(0, i, 9)] *= -1.0
        g[2, rng.integers(0, o, 3)] = 0.0
        if n == 1:
            h[2] = 0.0
        layers.append((signs, g.astype(np.float16), h.astype(np.float16)))
    x = synth.outlier_activations(rng, 1, widths[0])
    for pause in (0, -1):
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, pause)
        try:
            _check_stack(layers, [(0, 0, 1), (1, 1, 2), (2, 2, 3)], widths, x, 1, f"three paths, pause {pause}", True)
        finally:
            rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, -1)
