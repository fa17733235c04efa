"""The decoder block fused into the stack kernel (rb_block_prepare / rb_stack_run) against the
oracle, op by op and teacher-forced: the oracle recomputes every op from the buffers the GPU run
actually read (its input, and the residual stream it added)."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb
from helpers import TOL, random_layer, to_device_layer

pytestmark = pytest.mark.gpu

EPS = 1e-5


def build_block(which, n_layers, config, T, shrink=None, outliers=False, in_place=False, gain=None, K=2):
    """Layers, norm weights and the stack input of a Llama-shaped block stack: uniform signs,
    half-normal scales with a gain on g that keeps every op's output near RMS 1 for a normalised
    input, norm weights around 1 (a few negative, one zero)."""
    ops, shapes, widths, norms = synth.llama_block_stack(which, n_layers, in_place=in_place)
    m = (lambda w: shrink.get(w, w)) if shrink else (lambda w: w)
    widths = [m(w) for w in widths]
    layers = []
    for n, (name, out, inn) in enumerate(shapes):
        rng = synth.child_rng(config, 1, n)
        # y_i ~ g * sqrt(in) * rms(h) * rms(x): 0.02 * 0.02 * sqrt(in) per unit of gain
        g_gain = gain if gain is not None else 1.0 / (0.02 * 0.02 * np.sqrt(m(inn)))
        if name.endswith("down"):
            g_gain *= 2.0           # its input, silu(gate) * up, has RMS near 1/2
        layers.append(random_layer(rng, K, m(out), m(inn), gain=g_gain))
    norm_w = []
    for n, w in enumerate(norms):
        rng = synth.child_rng(config, 2, n)
        v = 1.0 + 0.2 * rng.standard_normal(m(w))
        v[rng.integers(0, m(w), 3)] *= -1.0
        v[rng.integers(0, m(w))] = 0.0
        norm_w.append(v.astype(np.float16))
    x0 = (synth.outlier_activations if outliers else synth.gaussian_activations)(synth.child_rng(config, 0), T, widths[0])
    return ops, widths, layers, norm_w, x0


def _op_tuples(ops):
    return [(o.layer, o.src, o.dst, o.norm, o.epilogue, o.aux) for o in ops]


def _run(ops, widths, layers, norm_w, x0, T, pause=-1, runs=1):
    dev_layers = [to_device_layer(*l) for l in layers]
    dev_norms = [torch.from_numpy(w).cuda() for w in norm_w]
    dev_bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    dev_bufs[0].copy_(torch.from_numpy(x0))
    block = rb.Block(dev_layers, dev_norms, EPS, _op_tuples(ops), dev_bufs, T)
    block.prepare()
    rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, pause)
    try:
        for _ in range(runs):
            block.run_prepared()
        torch.cuda.synchronize()
    finally:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, -1)
    assert rb.rb_last_path() == rb.RB_PATH_MX
    assert block.status() == rb.RB_OK, f"gave up: reason {block.gave_up()}"
    waited = block.waited()
    block.forget()
    return [b.cpu().numpy() for b in dev_bufs], waited, (dev_layers, dev_norms, dev_bufs)


def _check(ops, layers, norm_w, got, label):
    refs = oracle.block_forward(layers, norm_w, EPS, _op_tuples(ops), got, write_back=False)
    worst = 0.0
    for n, op in enumerate(ops):
        assert np.all(np.isfinite(got[op.dst])), op.name
        err = float(oracle.relative_l2(got[op.dst].astype(np.float64), refs[n]).max())
        worst = max(worst, err)
        assert err <= TOL, (label, op.name, err)
    print(f"  {label}: worst teacher-forced rel_l2={worst:.3e}", flush=True)
    return worst


SHRINK = {4096: 512, 11008: 1376}


@pytest.mark.parametrize("T", [1, 2, 3, 4])
def test_small_block_stack(T):
    """Three blocks at 1/8 width: normalised q/k/v and gate/up, gate times up, both residual
    additions, outlier channels in the stack input."""
    ops, widths, layers, norm_w, x0 = build_block("7b", 3, 40 + T, T, shrink=SHRINK, outliers=True)
    print(f"block stack at 1/8 width: {len(ops)} ops, T={T}", flush=True)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    _check(ops, layers, norm_w, got, f"small block stack T={T}")
    # the residual stream stays in range over the blocks
    assert 0.3 < float(np.sqrt((got[ops[-1].dst].astype(np.float64) ** 2).mean())) < 30.0


@pytest.mark.parametrize("T", [1, 4])
def test_full_width_7b_blocks(T):
    """Two blocks at the real 7B widths (688 row tiles of gate and of up: two or three per
    workgroup, meeting in the halves of the finishing wavefronts)."""
    ops, widths, layers, norm_w, x0 = build_block("7b", 2, 50 + T, T, outliers=True)
    print(f"two full-width 7B blocks, T={T}", flush=True)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    _check(ops, layers, norm_w, got, f"full-width 7B blocks T={T}")


def test_three_path_blocks_one_token():
    """The 3-bit variant: three paths in every layer, one token (the third path rides in the lanes
    of a second token), at 1/8 width over three blocks and at full 7B width."""
    ops, widths, layers, norm_w, x0 = build_block("7b", 3, 58, 1, shrink=SHRINK, outliers=True, K=3)
    print("three-path block stack at 1/8 width", flush=True)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, 1)
    _check(ops, layers, norm_w, got, "three-path small block stack")
    ops, widths, layers, norm_w, x0 = build_block("7b", 1, 59, 1, K=3)
    print("one full-width three-path 7B block", flush=True)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, 1)
    _check(ops, layers, norm_w, got, "three-path full-width block")
    # two tokens of three paths: not on this kernel
    ops, widths, layers, norm_w, x0 = build_block("7b", 1, 59, 2, shrink=SHRINK, K=3)
    dev_layers = [to_device_layer(*l) for l in layers]
    dev_norms = [torch.from_numpy(w).cuda() for w in norm_w]
    dev_bufs = [torch.zeros((2, w), dtype=torch.float16, device="cuda") for w in widths]
    with pytest.raises(rb.RabitError) as e:
        rb.Block(dev_layers, dev_norms, EPS, _op_tuples(ops), dev_bufs, 2).prepare()
    assert e.value.code == rb.RB_ERR_UNSUPPORTED


def test_one_13b_block():
    """13824 rows of gate and up: four row tiles per workgroup, every finishing slot in use."""
    ops, widths, layers, norm_w, x0 = build_block("13b", 1, 57, 1)
    print("one full-width 13B block, T=1", flush=True)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, 1)
    _check(ops, layers, norm_w, got, "13B block")


@pytest.mark.parametrize("T", [1, 2])
def test_block_stack_without_pause(T):
    """No pause between a workgroup's stores and its go: readers look for sums of squares,
    residual values and input tiles before they are written, and must wait for each."""
    ops, widths, layers, norm_w, x0 = build_block("7b", 4, 60 + T, T, shrink=SHRINK)
    print(f"block stack without pause, T={T}", flush=True)
    got, waited, _ = _run(ops, widths, layers, norm_w, x0, T, pause=0, runs=3)
    _check(ops, layers, norm_w, got, f"no pause T={T}")
    print(f"  tiles waited for: {waited}", flush=True)
    # and the same bits as with the built-in pacing
    again, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    for a, b in zip(got, again):
        assert np.array_equal(a, b)


def test_residual_stream_in_place():
    """The residual stream kept in one buffer (dst == aux) gives the bits of the run with a buffer
    per op."""
    T = 2
    ops, widths, layers, norm_w, x0 = build_block("7b", 3, 70, T, shrink=SHRINK)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    ops_ip, widths_ip, _, _, _ = build_block("7b", 3, 70, T, shrink=SHRINK, in_place=True)
    got_ip, _, _ = _run(ops_ip, widths_ip, layers, norm_w, x0, T)
    assert np.array_equal(got_ip[0], got[ops[-1].dst])
    # the other buffers (q, k, v, act of every block) too
    for a, b in zip(ops, ops_ip):
        if b.dst != 0:
            assert np.array_equal(got[a.dst], got_ip[b.dst]), a.name


def test_ragged_rows_and_plain_ops_in_a_block():
    """A block list that mixes plain ops with the fused ones; a dead-end op whose rows are not a
    multiple of 16; an op that adds a buffer written by an op it does not read."""
    T = 2
    rng = synth.child_rng(80, 0)
    d, f = 544, 1056
    shapes = [(300, d), (d, d), (d, d), (f, d), (f, d), (d, f), (d, d)]
    gains = [1.0 / (0.02 * 0.02 * np.sqrt(i)) for _, i in shapes]
    layers = [random_layer(synth.child_rng(80, 1, n), 2, o, i, gain=gn) for n, ((o, i), gn) in enumerate(zip(shapes, gains))]
    norm_w = [(1.0 + 0.1 * rng.standard_normal(d)).astype(np.float16)]
    widths = [d, 300, d, d, f, d, d]
    E = (rb.RB_EPI_NONE, rb.RB_EPI_ADD, rb.RB_EPI_SILU_MUL)

    class O:
        def __init__(self, name, layer, src, dst, norm, epilogue, aux):
            self.name, self.layer, self.src, self.dst, self.norm, self.epilogue, self.aux = name, layer, src, dst, norm, epilogue, aux
    ops = [O("ragged", 0, 0, 1, 0, E[0], -1),          # 300 rows, normalised input from outside
           O("plain", 1, 0, 2, -1, E[0], -1),          # no norm, no epilogue
           O("add_x", 2, 2, 3, -1, E[1], 0),           # adds the stack input
           O("gate_up", 3, 3, 4, 0, E[2], 4),
           O("down", 5, 4, 5, -1, E[1], 3),
           O("add_far", 6, 5, 6, 0, E[1], 2)]          # normalised input, adds what "plain" wrote
    x0 = synth.gaussian_activations(rng, T, d)
    got, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    _check(ops, layers, norm_w, got, "mixed block list")


def test_degenerate_inputs():
    """An all-zero token (its normalised input is zero, not NaN) next to an ordinary one; large
    activations (sums of squares beyond fp16's range stay in fp32)."""
    T = 2
    ops, widths, layers, norm_w, x0 = build_block("7b", 1, 90, T, shrink=SHRINK)
    x0 = x0.copy()
    x0[0, :] = 0.0
    x0[1, :] = (x0[1, :].astype(np.float64) * 300.0).astype(np.float16)      # sum of squares ~ 5e7
    got, _, _ = _run(ops, widths, layers, norm_w, x0, T)
    refs = oracle.block_forward(layers, norm_w, EPS, _op_tuples(ops), got, write_back=False)
    for n, op in enumerate(ops):
        assert np.all(np.isfinite(got[op.dst])), op.name
        if op.src == 0:
            assert np.all(got[op.dst][0] == 0), op.name          # q, k, v of the zero token
        err = oracle.relative_l2(got[op.dst].astype(np.float64), refs[n])
        assert float(err[1]) <= TOL, (op.name, err)
        ref0 = np.abs(refs[n][0]).max()
        assert float(err[0]) <= TOL or ref0 == 0.0, (op.name, err)


def test_separate_kernels_against_the_oracle():
    """rb_rmsnorm, rb_silu_mul, rb_add: one rounding to fp16 of the fp32 result."""
    rng = synth.child_rng(95, 0)
    T, n = 3, 1376
    x = synth.outlier_activations(rng, T, n)
    w = (1.0 + 0.2 * rng.standard_normal(n)).astype(np.float16)
    y = rb.rb_rmsnorm(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), EPS).cpu().numpy()
    ref = oracle.rmsnorm(x, w, EPS)
    assert float(oracle.relative_l2(y, ref).max()) <= 5e-4
    np.testing.assert_allclose(y.astype(np.float64), ref, rtol=2.0 ** -10, atol=1e-7)
    a = (rng.standard_normal((T, n)) * 3).astype(np.float16)
    b = rng.standard_normal((T, n)).astype(np.float16)
    s = rb.rb_silu_mul(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()).cpu().numpy()
    np.testing.assert_allclose(s.astype(np.float64), oracle.silu(a) * b.astype(np.float64), rtol=2.0 ** -10, atol=1e-7)
    c = rb.rb_add(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()).cpu().numpy()
    assert np.array_equal(c, (a.astype(np.float64) + b.astype(np.float64)).astype(np.float16))


def test_fused_block_against_op_by_op_kernels():
    """The same block run op by op (rb_rmsnorm, rb_layer_stack, rb_silu_mul, rb_add): both
    routes meet the oracle; they differ from each other only by the fp16 roundings of the
    intermediates the fused route never stores."""
    T = 1
    ops, widths, layers, norm_w, x0 = build_block("7b", 1, 97, T, shrink=SHRINK)
    got, _, (dev_layers, dev_norms, _) = _run(ops, widths, layers, norm_w, x0, T)
    x = torch.from_numpy(x0).cuda()
    n1 = rb.rb_rmsnorm(x, dev_norms[0], EPS)
    q, k, v = (rb.rb_linear_gemm(dev_layers[i], n1) for i in range(3))
    x1 = rb.rb_add(rb.rb_linear_gemm(dev_layers[3], v), x)
    n2 = rb.rb_rmsnorm(x1, dev_norms[1], EPS)
    act = rb.rb_silu_mul(rb.rb_linear_gemm(dev_layers[4], n2), rb.rb_linear_gemm(dev_layers[5], n2))
    x2 = rb.rb_add(rb.rb_linear_gemm(dev_layers[6], act), x1)
    torch.cuda.synchronize()
    for name, a, b in (("q", q, got[1]), ("v", v, got[3]), ("x1", x1, got[4]), ("act", act, got[5]), ("x2", x2, got[6])):
        err = float(oracle.relative_l2(a.cpu().numpy(), b.astype(np.float64)).max())
        print(f"  {name}: op-by-op vs fused rel_l2={err:.3e}", flush=True)
        assert err <= 3e-3, name


def test_block_beyond_the_fused_kernel_is_refused():
    ops, widths, layers, norm_w, x0 = build_block("7b", 1, 99, 5, shrink=SHRINK)
    dev_layers = [to_device_layer(*l) for l in layers]
    dev_norms = [torch.from_numpy(w).cuda() for w in norm_w]
    dev_bufs = [torch.zeros((5, w), dtype=torch.float16, device="cuda") for w in widths]
    block = rb.Block(dev_layers, dev_norms, EPS, _op_tuples(ops), dev_bufs, 5)
    with pytest.raises(rb.RabitError) as e:
        block.prepare()
    assert e.value.code == rb.RB_ERR_UNSUPPORTED


@pytest.mark.parametrize("T", [1, 2, 4])
def test_full_7b_block_stack_without_pause(T):
    """The 32-block stack as bench.py builds it with the hand-over pause set to zero: at full width
    every wavefront that waits looks again while all the others do the same and the producers still
    store.  Same bits as the paced run, no wait given up."""
    import bench
    ops, layers, norms, bufs, x0, op_list, _ = bench.build_block_stack(rb, synth, torch, "7b", T)
    block = rb.Block(layers, norms, 1e-5, op_list, bufs, T)
    block.prepare()
    bufs[0].copy_(x0)
    block.run_prepared()
    torch.cuda.synchronize()
    assert block.status() == rb.RB_OK, f"gave up: reason {block.gave_up()}"
    paced = [b.clone() for b in bufs]
    before = block.waited()
    try:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, 0)
        print(f"no hand-over pause, full 7B-shaped block stack, T={T}", flush=True)
        for run in range(4):
            for b in bufs[1:]:
                b.zero_()
            bufs[0].copy_(x0)
            block.run_prepared()
            torch.cuda.synchronize()
            assert block.status() == rb.RB_OK, f"run {run} gave up: reason {block.gave_up()}"
            bad = [n for n, (a, b) in enumerate(zip(paced, bufs)) if not torch.equal(a, b)]
            assert not bad, (run, bad[:5])
    finally:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, -1)
    print(f"  tiles read again: {block.waited() - before}", flush=True)
    block.forget()


def test_full_7b_block_stack_as_benchmarked_sampled_outputs():
    """The 32-block stack exactly as bench.py builds and times it (residual stream in one buffer):
    status clean, and bit for bit the run of the same ops with a buffer per op, whose sampled rows
    (first, a middle and the last block) are recomputed by the oracle from the stored bits and the
    buffers that run read."""
    import bench
    T = 1
    ops_ip, layers, norms, bufs_ip, x0, list_ip, packed = bench.build_block_stack(rb, synth, torch, "7b", T)
    ops, layers2, norms2, bufs, x0b, op_list, _ = bench.build_block_stack(rb, synth, torch, "7b", T, in_place=False)
    assert len(ops) == 192 and len(layers) == 224 and packed == 1619001344
    assert torch.equal(x0, x0b) and all(torch.equal(a.bits, b.bits) for a, b in zip(layers, layers2))
    results = []
    for name, o_list, bb in (("in place", list_ip, bufs_ip), ("a buffer per op", op_list, bufs)):
        print(f"full 7B-shaped block stack, {name}", flush=True)
        block = rb.Block(layers, norms, 1e-5, o_list, bb, T)
        block.prepare()
        for run in range(2):                        # scratch state must not leak between runs
            bb[0].copy_(x0)
            block.run_prepared()
            torch.cuda.synchronize()
            assert rb.rb_last_path() == rb.RB_PATH_MX and block.status() == rb.RB_OK
            results.append([b.clone() for b in bb])
        block.forget()
    for a, b in zip(results[0], results[1]):
        assert torch.equal(a, b)
    for a, b in zip(results[2], results[3]):
        assert torch.equal(a, b)
    assert torch.equal(results[0][0], results[2][ops[-1].dst])           # the residual stream after the last block
    for a, b in zip(ops, ops_ip):
        if b.dst != 0:
            assert torch.equal(results[2][a.dst], results[0][b.dst]), a.name
    # sampled rows against the oracle
    pick = np.random.default_rng(77)
    host = [b.cpu().numpy() for b in bufs]
    worst = 0.0

    def rows_of(L, rows):
        packed_words = rb.rb_unpack_native(L.bits.cpu().numpy().view(np.uint32), 2, L.out, L.inn)
        return rb.rb_unpack(packed_words[:, rows, :]), L.g.cpu().numpy()[:, rows], L.h.cpu().numpy()
    for blk in (0, 15, 31):
        for op in ops[6 * blk: 6 * blk + 6]:
            L = layers[op.layer]
            rows = np.unique(pick.integers(0, L.out, size=40))
            x = host[op.src].astype(np.float64)
            if op.norm >= 0:
                x = oracle.rmsnorm(x, norms[op.norm].cpu().numpy(), 1e-5)
            ref = oracle.forward(*rows_of(L, rows), x)
            if op.epilogue == rb.RB_EPI_SILU_MUL:
                ref = oracle.silu(ref) * oracle.forward(*rows_of(layers[op.aux], rows), x)
            elif op.epilogue == rb.RB_EPI_ADD:
                ref = ref + host[op.aux].astype(np.float64)[:, rows]
            got = host[op.dst].astype(np.float64)[:, rows]
            assert np.all(np.isfinite(got)) and np.any(got != 0), op.name
            err = float(oracle.relative_l2(got, ref).max())
            worst = max(worst, err)
            assert err <= TOL, (op.name, err)
    print(f"  worst sampled rel_l2={worst:.3e}", flush=True)
