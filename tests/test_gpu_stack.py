"""rb_layer_stack vs the oracle, op by op.  Over 100+ dependent fp16-rounded
ops the two implementations drift apart by rounding alone, so parity is
teacher-forced: the oracle recomputes every op from the input the GPU run
actually used, and that op's output must agree to the usual tolerance."""
import sys

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb
from helpers import TOL, build_stack, to_device_layer, random_layer

pytestmark = pytest.mark.gpu

DEFAULT_PAUSE = -1          # the kernel's built-in timing (rb_stack_set_option)


def _run_and_check(ops, widths, layers, bufs0, T, label, prepared=False):
    dev_layers = [to_device_layer(*l) for l in layers]
    dev_bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    dev_bufs[0].copy_(torch.from_numpy(bufs0[0]))
    op_list = [(n, op.src, op.dst) for n, op in enumerate(ops)]
    print(f"{label}: {len(ops)} ops, T={T}, prepared={prepared}", flush=True)
    if prepared:
        stack = rb.Stack(dev_layers, op_list, dev_bufs, T)
        stack.prepare()
        stack.run_prepared()
        torch.cuda.synchronize()
        assert rb.rb_last_path() == (rb.RB_PATH_MX if T < 8 else rb.RB_PATH_BATCH)
        assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
        stack.forget()
    else:
        rb.rb_layer_stack(dev_layers, op_list, dev_bufs, T)
    torch.cuda.synchronize()
    # a stack of 3..16 tokens runs as token pairs on the fused kernel or on the small-batch kernel,
    # a single call on the many-token kernel
    same_kernel = T <= 2 or T > 16
    got = [b.cpu().numpy() for b in dev_bufs]
    forced = [got[op.src] for op in ops]
    refs = oracle.stack_forward(layers, op_list, [None] * len(widths), forced_inputs=forced)
    worst = 0.0
    for n, op in enumerate(ops):
        assert np.all(np.isfinite(got[op.dst])), op.name
        err = float(oracle.relative_l2(got[op.dst].astype(np.float64), refs[n]).max())
        worst = max(worst, err)
        assert err <= TOL, (op.name, err)
        # the op must equal the single-layer call on the same input
        y1 = rb.rb_linear_gemm(dev_layers[n], dev_bufs[op.src])
        if same_kernel:
            assert torch.equal(y1, dev_bufs[op.dst]), op.name
        else:
            assert float(oracle.relative_l2(y1.cpu().numpy().astype(np.float64), refs[n]).max()) <= TOL, op.name
    # free-running drift against the oracle's own chain: information only
    drift = float(oracle.relative_l2(got[ops[-1].dst].astype(np.float64),
                                     bufs0[ops[-1].dst].astype(np.float64)).max())
    print(f"  worst teacher-forced rel_l2={worst:.3e}; end-to-end drift={drift:.3e}", flush=True)
    sys.stdout.flush()


def test_small_stack_derived_weights_three_blocks():
    shrink = {4096: 512, 11008: 1376}
    ops, widths, layers, bufs = build_stack("7b", 3, 2, 1, derived=True, shrink=shrink)
    _run_and_check(ops, widths, layers, bufs, 1, "7B-dataflow stack at 1/8 width, derived")


def test_one_full_width_7b_block_derived():
    ops, widths, layers, bufs = build_stack("7b", 1, 2, 1, derived=True)
    _run_and_check(ops, widths, layers, bufs, 1, "one 7B-shaped block, derived")


@pytest.mark.parametrize("T", [2, 4, 16])
def test_small_stack_batched_with_outliers(T):
    shrink = {4096: 512, 11008: 1376}
    # uniform-sign layers with 0.02-scale g and h: a gain on g keeps activations near RMS 1
    ops, widths, layers, bufs = build_stack("7b", 2, 3, T, derived=False, shrink=shrink, outliers=True,
                                            gain=100.0)
    _run_and_check(ops, widths, layers, bufs, T, "batched small stack")


@pytest.mark.parametrize("T", [3, 8, 16])
def test_prepared_small_batches(T):
    """rb_stack_prepare / rb_stack_run at 3..16 tokens (token pairs on the fused kernel below 8
    tokens, the small-batch kernel from 8 on), every op checked against the oracle."""
    shrink = {4096: 512, 11008: 1376}
    ops, widths, layers, bufs = build_stack("7b", 2, 5, T, derived=False, shrink=shrink, outliers=True,
                                            gain=100.0)
    _run_and_check(ops, widths, layers, bufs, T, "prepared small batch", prepared=True)


def test_one_13b_block_derived():
    ops, widths, layers, bufs = build_stack("13b", 1, 4, 1, derived=True)
    _run_and_check(ops, widths, layers, bufs, 1, "one 13B-shaped block, derived")


def test_prepare_once_run_many_tokens():
    """rb_stack_prepare + rb_stack_run: one set-up, then one run per token; every run must equal
    rb_layer_stack on the same input bit for bit."""
    shrink = {4096: 512, 11008: 1376}
    ops, widths, layers, bufs = build_stack("7b", 2, 2, 1, derived=False, shrink=shrink, gain=100.0)
    dev_layers = [to_device_layer(*l) for l in layers]
    dev_bufs = [torch.zeros((1, w), dtype=torch.float16, device="cuda") for w in widths]
    ref_bufs = [torch.zeros((1, w), dtype=torch.float16, device="cuda") for w in widths]
    op_list = [(n, op.src, op.dst) for n, op in enumerate(ops)]
    stack = rb.Stack(dev_layers, op_list, dev_bufs, 1)
    stack.prepare()
    for token in range(4):
        x = synth.gaussian_activations(synth.child_rng(2, 50, token), 1, widths[0])
        dev_bufs[0].copy_(torch.from_numpy(x)); ref_bufs[0].copy_(torch.from_numpy(x))
        print(f"prepared stack, token {token}", flush=True)
        stack.run_prepared()
        rb.rb_layer_stack(dev_layers, op_list, ref_bufs, 1)
        torch.cuda.synchronize()
        for a, b in zip(dev_bufs, ref_bufs):
            assert torch.equal(a, b)
        last = oracle.forward(*layers[-1], dev_bufs[ops[-1].src].cpu().numpy())
        assert oracle.relative_l2(dev_bufs[ops[-1].dst].cpu().numpy().astype(np.float64), last).max() <= TOL
    assert stack.status() == rb.RB_OK                 # no run gave up a hand-over wait
    stack.forget()
    assert stack.status() == rb.RB_ERR_WORKSPACE
    with pytest.raises(rb.RabitError):
        stack.run_prepared()


def test_non_finite_activation_propagates_and_ends():
    """An infinity in the input must come out as non-finite outputs of every dependent op, at once:
    the flag-free hand-over tells "not written yet" from data by a byte pattern that a NaN term
    could otherwise take, and a wait on it would only end at its (long) bound with RB_ERR_HANDOVER."""
    shrink = {4096: 512, 11008: 1376}
    ops, widths, layers, bufs = build_stack("7b", 1, 7, 1, derived=False, shrink=shrink, gain=100.0)
    dev_layers = [to_device_layer(*l) for l in layers]
    op_list = [(n, op.src, op.dst) for n, op in enumerate(ops)]
    dev_bufs = [torch.zeros((1, w), dtype=torch.float16, device="cuda") for w in widths]
    x = torch.from_numpy(bufs[0]).clone()
    x[0, 5] = float("inf")
    x[0, 77] = float("nan")
    dev_bufs[0].copy_(x)
    stack = rb.Stack(dev_layers, op_list, dev_bufs, 1)
    stack.prepare()
    print("non-finite input through a dependent stack", flush=True)
    stack.run_prepared()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    stack.forget()
    for op in ops:
        assert not torch.isfinite(dev_bufs[op.dst]).any(), op.name


@pytest.mark.parametrize("T", [1, 2, 3, 4])
def test_requests_ahead_of_the_writes_are_caught(T):
    """With the hand-over pause set to zero every workgroup asks for a phase's inputs the moment its
    own part is stored, so many input tiles are requested before the other workgroups have written
    them.  The consumer must notice every such tile (the 'not written yet' pattern), wait for it
    and read it again: same bits as the normally paced run, clean status, every kernel ends by
    itself."""
    shrink = {4096: 1024, 11008: 2752}
    ops, widths, layers, bufs = build_stack("7b", 2, 8, T, derived=False, shrink=shrink, gain=100.0)
    dev_layers = [to_device_layer(*l) for l in layers]
    op_list = [(n, op.src, op.dst) for n, op in enumerate(ops)]
    results, waited = [], []
    try:
        for pause in (None, 0, 200):
            if pause is not None:
                rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, pause)
            dev_bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
            print(f"hand-over pause {pause}, T={T}", flush=True)
            stack = rb.Stack(dev_layers, op_list, dev_bufs, T)
            stack.prepare()
            runs = []
            for token in range(6):
                x = synth.gaussian_activations(synth.child_rng(2, 61, token), T, widths[0])
                dev_bufs[0].copy_(torch.from_numpy(x))
                stack.run_prepared()
                torch.cuda.synchronize()
                runs.append([b.clone() for b in dev_bufs])
            assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
            waited.append(stack.waited())
            print(f"  tiles read again: {waited[-1]}", flush=True)
            stack.forget()
            results.append(runs)
    finally:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, DEFAULT_PAUSE)
    assert waited[1] > 0                                     # the unpaced run did exercise the waits
    for other in results[1:]:
        for run_a, run_b in zip(results[0], other):
            for a, b in zip(run_a, run_b):
                assert torch.equal(a, b)
    last = oracle.forward(*layers[-1], results[0][-1][ops[-1].src].cpu().numpy())
    assert oracle.relative_l2(results[0][-1][ops[-1].dst].cpu().numpy().astype(np.float64), last).max() <= TOL


def test_independent_ops_need_no_hand_over():
    """Ops that all read buffers nobody writes (the small-batch recipe: every op has its own
    input) run in one launch without waiting on each other."""
    rng = synth.child_rng(3, 77)
    shapes = [(512, 512), (1376, 512), (512, 1376), (512, 512), (1376, 512)]
    layers = [random_layer(rng, 2, o, i) for (o, i) in shapes]
    xs = [synth.outlier_activations(rng, 2, i) for (_, i) in shapes]
    dev_layers = [to_device_layer(*l) for l in layers]
    bufs = [torch.from_numpy(x).cuda() for x in xs] + \
           [torch.zeros((2, o), dtype=torch.float16, device="cuda") for (o, _) in shapes]
    op_list = [(n, n, len(shapes) + n) for n in range(len(shapes))]
    print("independent ops, T=2", flush=True)
    rb.rb_layer_stack(dev_layers, op_list, bufs, 2)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX
    for n in range(len(shapes)):
        ref = oracle.forward(*layers[n], xs[n])
        assert oracle.relative_l2(bufs[len(shapes) + n].cpu().numpy().astype(np.float64), ref).max() <= TOL


def test_full_7b_stack_as_benchmarked_sampled_outputs():
    """The 224-op 7B-shaped stack exactly as bench.py builds and times it (prepared, one launch per
    token, signs drawn on the device in native order).  For the ops of the first, a middle and the
    last block, 48 sampled rows are recomputed by the oracle from the unpacked rows and from the
    input the GPU run actually used; a second run over the same input must repeat the first bit
    for bit (flags and scratch are cleared correctly between launches)."""
    import bench
    ops, layers, bufs, op_list, packed_bytes = bench.build_stack(rb, synth, torch, "7b", 1)
    assert len(ops) == 224 and packed_bytes == 1619001344
    stack = rb.Stack(layers, op_list, bufs, 1)
    stack.prepare()
    print("full 7B-shaped stack, prepared, run 1", flush=True)
    stack.run_prepared()
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX
    first = [b.clone() for b in bufs]
    print("full 7B-shaped stack, run 2", flush=True)
    stack.run_prepared()
    torch.cuda.synchronize()
    for a, b in zip(first, bufs):
        assert torch.equal(a, b)
    stack.forget()
    pick = np.random.default_rng(11)
    worst = 0.0
    for blk in (0, 15, 31):
        for n in range(7 * blk, 7 * blk + 7):
            op, L = ops[n], layers[n]
            y = bufs[op.dst].cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(y)) and np.any(y != 0), op.name
            native = L.bits.cpu().numpy().view(np.uint32)
            packed = rb.rb_unpack_native(native, 2, L.out, L.inn)
            rows = np.unique(pick.integers(0, L.out, size=48))
            S = rb.rb_unpack(packed[:, rows, :])
            g = L.g.cpu().numpy()[:, rows]
            ref = oracle.forward(S, g, L.h.cpu().numpy(), bufs[op.src].cpu().numpy())
            err = float(oracle.relative_l2(y[:, rows], ref).max())
            worst = max(worst, err)
            assert err <= TOL, (op.name, err)
    print(f"  worst sampled rel_l2={worst:.3e}", flush=True)


def test_three_path_layers_in_a_stack():
    """K = 3 layers in a stack of two tokens run on the small-batch matrix-core kernel (three right
    operands per 128 columns), every op checked against the oracle."""
    rng = synth.child_rng(3, 88)
    shapes = [(192, 256), (320, 192), (192, 320)]              # x -> a -> b -> c
    layers = []
    for (o, i) in shapes:
        W = rng.standard_normal((o, i)) / np.sqrt(i)
        signs, g, h, _ = oracle.derive(W, 3)
        layers.append((signs, g, h))
    T = 2
    x = synth.gaussian_activations(rng, T, 256)
    dev_layers = [to_device_layer(*l) for l in layers]
    bufs = [torch.from_numpy(x).cuda()] + [torch.zeros((T, o), dtype=torch.float16, device="cuda") for (o, _) in shapes]
    op_list = [(0, 0, 1), (1, 1, 2), (2, 2, 3)]
    print("K=3 stack of three ops, T=2", flush=True)
    rb.rb_layer_stack(dev_layers, op_list, bufs, T)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_BATCH
    for n, (l, s, d) in enumerate(op_list):
        ref = oracle.forward(*layers[l], bufs[s].cpu().numpy())
        assert oracle.relative_l2(bufs[d].cpu().numpy().astype(np.float64), ref).max() <= TOL, n


def test_hand_over_at_full_scale_many_tokens():
    """Every op of the full 7B-shaped stack, over 40 tokens, against the single-op kernel on the
    input that op actually read: the two share every rounding step, so any operand that a compute
    unit picked up before its producer had finished shows up as a mismatch."""
    import bench
    ops, layers, bufs, op_list, _ = bench.build_stack(rb, synth, torch, "7b", 1)
    stack = rb.Stack(layers, op_list, bufs, 1)
    stack.prepare()
    gen = torch.Generator(device="cuda"); gen.manual_seed(77)
    ys = [torch.empty_like(bufs[op.dst]) for op in ops]
    ws = rb.binding._workspace(layers[:7], 1, bufs[0].device)       # all seven shapes
    for token in range(40):
        bufs[0].copy_(torch.randn(1, ops[0].inn, device="cuda", generator=gen).half())
        if token % 10 == 0:
            print(f"full stack, token {token}", flush=True)
        stack.run_prepared()
        for n, op in enumerate(ops):
            rb.rb_linear_gemm(layers[n], bufs[op.src], Y=ys[n], workspace=ws)
        torch.cuda.synchronize()
        bad = [op.name for n, op in enumerate(ops) if not torch.equal(ys[n], bufs[op.dst])]
        assert not bad, (token, bad[:5])
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    stack.forget()


# ------------------------------------------------------------------------------------------
# The configurations the benchmark times, at the widths and through the entry points it uses
# ------------------------------------------------------------------------------------------
def _sampled_rows_check(rb_mod, ops, layers, bufs, op_numbers, rows_per_op, seed):
    """Recompute sampled rows of the given ops with the oracle from the unpacked stored bits and the
    input the GPU run used; returns the worst per-vector relative error."""
    pick = np.random.default_rng(seed)
    worst = 0.0
    for n in op_numbers:
        op, L = ops[n], layers[n]
        y = bufs[op.dst].cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(y)) and np.any(y != 0), op.name
        native = L.bits.cpu().numpy().view(np.uint32)
        packed = rb_mod.rb_unpack_native(native, 2, L.out, L.inn)
        rows = np.unique(pick.integers(0, L.out, size=rows_per_op))
        S = rb_mod.rb_unpack(packed[:, rows, :])
        g = L.g.cpu().numpy()[:, rows]
        ref = oracle.forward(S, g, L.h.cpu().numpy(), bufs[op.src].cpu().numpy())
        err = float(oracle.relative_l2(y[:, rows], ref).max())
        worst = max(worst, err)
        assert err <= TOL, (op.name, err)
    return worst


@pytest.mark.parametrize("T,runs", [(1, 10000), (3, 3000)])
def test_determinism_canary_and_hand_over_stress(T, runs):
    """The 7B-shaped stack as the benchmark builds it, run after run on the same input: the first
    100 runs must reproduce every buffer bit for bit, and after thousands of runs (every one of
    them 128 hand-overs between all compute units) the outputs are still those bits and no wait
    was ever given up."""
    import bench
    ops, layers, bufs, op_list, _ = bench.build_stack(rb, synth, torch, "7b", T)
    stack = rb.Stack(layers, op_list, bufs, T)
    stack.prepare()
    stack.run_prepared()
    torch.cuda.synchronize()
    first = [b.clone() for b in bufs]
    print(f"determinism canary, T={T}: 100 runs, every buffer", flush=True)
    for run in range(100):
        stack.run_prepared()
        torch.cuda.synchronize()
        bad = [n for n, (a, b) in enumerate(zip(first, bufs)) if not torch.equal(a, b)]
        assert not bad, (run, bad[:5])
    print(f"hand-over stress, T={T}: {runs} runs", flush=True)
    for run in range(runs):
        stack.run_prepared()
        if run % 1000 == 999:
            torch.cuda.synchronize()
            assert torch.equal(first[ops[-1].dst], bufs[ops[-1].dst]), run
            print(f"  {run + 1} runs", flush=True)
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    bad = [n for n, (a, b) in enumerate(zip(first, bufs)) if not torch.equal(a, b)]
    assert not bad, bad[:5]
    stack.forget()


@pytest.mark.parametrize("T,K", [(1, 2), (2, 2), (3, 2), (4, 2), (1, 3)])
def test_unpaced_hand_over_on_the_full_stack(T, K):
    """The 7B-shaped stack as the benchmark builds it with the hand-over pause set to zero: at every
    one of its 128 hand-overs nearly every wavefront asks for its inputs before they are written and
    has to look again while the producers still store.  Same bits as the paced run, no wait given
    up.  (With four tokens a waiting wavefront used to fetch its whole 8 KB tile with every look;
    at this width those looks kept the second store of the producers' row tiles from landing until
    the waits were given up.)"""
    import bench
    ops, layers, bufs, op_list, _ = bench.build_stack(rb, synth, torch, "7b", T, K=K)
    stack = rb.Stack(layers, op_list, bufs, T)
    stack.prepare()
    stack.run_prepared()
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    paced = [b.clone() for b in bufs]
    waited_before = stack.waited()
    try:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, 0)
        print(f"no hand-over pause, full 7B-shaped stack, T={T}, K={K}", flush=True)
        for run in range(5):
            for b in bufs[1:]:
                b.zero_()
            stack.run_prepared()
            torch.cuda.synchronize()
            assert stack.status() == rb.RB_OK, f"run {run} gave up: reason {stack.gave_up()}"
            bad = [n for n, (a, b) in enumerate(zip(paced, bufs)) if not torch.equal(a, b)]
            assert not bad, (run, bad[:5])
    finally:
        rb.rb_stack_set_option(rb.RB_OPT_HANDOVER_PAUSE, DEFAULT_PAUSE)
    waited = stack.waited() - waited_before
    print(f"  tiles read again: {waited}", flush=True)
    assert waited > 100000                                   # the unpaced runs did exercise the waits
    stack.forget()


@pytest.mark.parametrize("T", [2, 3, 4])
def test_one_full_width_7b_block_small_batches_chained(T):
    """The two- and four-token forms of the fused kernel (three tokens use the layout of four) at
    the real 7B widths (43 column tiles, 688 row tiles, two or three per workgroup), ops in
    dependency order, outlier channels in the stack input."""
    ops, widths, layers, bufs = build_stack("7b", 1, 3, T, derived=False, outliers=True, gain=100.0)
    _run_and_check(ops, widths, layers, bufs, T, f"one full-width 7B block, T={T}, chained", prepared=True)


@pytest.mark.parametrize("T", [2, 4, 8, 16])
def test_full_width_7b_block_small_batches_own_inputs(T):
    """The small-batch workload as it is defined and timed: the seven matrices of a 7B-shaped
    block at full width, every op on an input buffer of its own (N(0,1) with 1 % outlier channels
    times 20), through rb_stack_prepare / rb_stack_run.  Every output element is checked."""
    ops, _ = synth.llama_stack("7b", 1)
    rng = synth.child_rng(3, 300 + T)
    layers = [random_layer(rng, 2, op.out, op.inn) for op in ops]
    xs = [synth.outlier_activations(rng, T, op.inn) for op in ops]
    dev_layers = [to_device_layer(*l) for l in layers]
    bufs = [torch.from_numpy(x).cuda() for x in xs] + \
           [torch.zeros((T, op.out), dtype=torch.float16, device="cuda") for op in ops]
    op_list = [(n, n, len(ops) + n) for n in range(len(ops))]
    print(f"full-width block, own inputs, T={T}", flush=True)
    stack = rb.Stack(dev_layers, op_list, bufs, T)
    stack.prepare()
    stack.run_prepared()
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    first = [b.clone() for b in bufs]
    stack.run_prepared()                                 # scratch state must not leak between runs
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    stack.forget()
    for a, b in zip(first, bufs):
        assert torch.equal(a, b)
    worst = 0.0
    for n, op in enumerate(ops):
        ref = oracle.forward(*layers[n], xs[n])
        err = float(oracle.relative_l2(bufs[len(ops) + n].cpu().numpy().astype(np.float64), ref).max())
        worst = max(worst, err)
        assert err <= TOL, (op.name, T, err)
    print(f"  worst rel_l2={worst:.3e}", flush=True)


def test_full_13b_stack_as_benchmarked_sampled_outputs():
    """The 280-op 13B-shaped stack exactly as bench.py builds and times it: sampled rows of the
    first, a middle and the last block against the oracle, a second run bit-identical, status clean."""
    import bench
    ops, layers, bufs, op_list, packed_bytes = bench.build_stack(rb, synth, torch, "13b", 1)
    assert len(ops) == 280 and packed_bytes == 3171942400
    stack = rb.Stack(layers, op_list, bufs, 1)
    stack.prepare()
    print("full 13B-shaped stack, prepared, run 1", flush=True)
    stack.run_prepared()
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    first = [b.clone() for b in bufs]
    print("full 13B-shaped stack, run 2", flush=True)
    stack.run_prepared()
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    for a, b in zip(first, bufs):
        assert torch.equal(a, b)
    stack.forget()
    picked = [n for blk in (0, 20, 39) for n in range(7 * blk, 7 * blk + 7)]
    worst = _sampled_rows_check(rb, ops, layers, bufs, picked, 40, seed=13)
    print(f"  worst sampled rel_l2={worst:.3e}", flush=True)


# ------------------------------------------------------------------------------------------
# Degenerate scales and extreme activations on the matrix-core decode kernels
# ------------------------------------------------------------------------------------------
def _edge_layer(rng, out, inn, zero_path=None):
    """Scales with negative and exactly-zero entries (Section 4.1 puts no sign constraint on g, h);
    optionally one path whose input scales are all zero."""
    signs = synth.uniform_signs(rng, 2, out, inn)
    g = (rng.standard_normal((2, out)) * 0.05)
    h = (rng.standard_normal((2, inn)) * 0.05)
    g[:, rng.choice(out, size=max(1, out // 16), replace=False)] = 0.0
    h[:, rng.choice(inn, size=max(1, inn // 16), replace=False)] = 0.0
    g[1] *= 0.3
    h[1] *= 0.3
    if zero_path is not None:
        h[zero_path] = 0.0
    return signs, g.astype(np.float16), h.astype(np.float16)


def _edge_activations(rng, T, inn):
    """N(0,1) with 1 % outlier channels, a few entries at the ends of the fp16 range (+-65504),
    fp16 subnormals and exact zeros."""
    x = synth.outlier_activations(rng, T, inn).astype(np.float64)
    idx = rng.choice(inn, size=12, replace=False)
    x[:, idx[0:2]] = 65504.0
    x[:, idx[2:4]] = -65504.0
    x[:, idx[4:8]] = 3.0e-7 * np.array([1, -1, 2, -3])          # subnormal in fp16
    x[:, idx[8:12]] = 0.0
    return x.astype(np.float16)


@pytest.mark.parametrize("zero_path", [None, 0, 1])
def test_single_call_decode_kernel_with_degenerate_scales_and_extreme_inputs(zero_path):
    out, inn = 272, 4096 + 256
    rng = synth.child_rng(0, 400, 9 if zero_path is None else zero_path)
    signs, g, h = _edge_layer(rng, out, inn, zero_path)
    x = _edge_activations(rng, 1, inn)
    L = to_device_layer(signs, g, h)
    print(f"edge cases, single call, zero_path={zero_path}", flush=True)
    y = rb.rb_linear_gemv(L, torch.from_numpy(x[0]).cuda())
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX
    ref = oracle.forward(signs, g, h, x)
    got = y.cpu().numpy().astype(np.float64)[None]
    assert np.all(np.isfinite(got))
    err = float(oracle.relative_l2(got, ref)[0])
    print(f"  rel_l2={err:.3e}", flush=True)
    assert err <= TOL
    # rows whose output scales are both zero give exactly zero
    dead = np.where((g[0] == 0) & (g[1] == 0))[0]
    assert dead.size > 0 and np.all(got[0, dead] == 0.0)


@pytest.mark.parametrize("T", [1, 2])
def test_stack_decode_kernel_with_degenerate_scales_and_extreme_inputs(T):
    """Three dependent ops through the persistent kernel.  The first op is fed from outside with
    extreme activations; its output scales make some of its outputs large (thousands) and others
    fp16-subnormal, and those feed an op whose input scales contain negatives, zeros and one
    all-zero path, whose output feeds a third."""
    rng = synth.child_rng(0, 410 + T)
    d0, d1, d2, d3 = 1024 + 32, 576, 800, 272
    l1 = _edge_layer(rng, d1, d0)
    g1 = l1[1].astype(np.float64)
    g1[:, : d1 // 8] *= 200.0                        # some outputs in the thousands
    g1[:, d1 // 8: d1 // 4] *= 1e-5                  # some outputs subnormal in fp16
    l1 = (l1[0], g1.astype(np.float16), l1[2])
    l2 = _edge_layer(rng, d2, d1, zero_path=1)
    l3 = _edge_layer(rng, d3, d2, zero_path=0)
    layers = [l1, l2, l3]
    x = _edge_activations(rng, T, d0)
    x[x == 65504.0] = 2000.0                         # keep the first op's outputs finite in fp16
    x[x == -65504.0] = -2000.0
    dev_layers = [to_device_layer(*l) for l in layers]
    widths = [d0, d1, d2, d3]
    dev_bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    dev_bufs[0].copy_(torch.from_numpy(x))
    op_list = [(0, 0, 1), (1, 1, 2), (2, 2, 3)]
    print(f"edge cases, three dependent ops, T={T}", flush=True)
    stack = rb.Stack(dev_layers, op_list, dev_bufs, T)
    stack.prepare()
    stack.run_prepared()
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_MX and stack.status() == rb.RB_OK
    stack.forget()
    got = [b.cpu().numpy() for b in dev_bufs]
    y1 = got[1].astype(np.float64)
    assert np.all(np.isfinite(y1)) and np.abs(y1).max() > 1000.0
    assert np.any((np.abs(y1) < 6.1e-5) & (y1 != 0)), "no fp16-subnormal activation reached the second op"
    for n, (l, s, d) in enumerate(op_list):
        ref = oracle.forward(*layers[l], got[s])
        err = float(oracle.relative_l2(got[d].astype(np.float64), ref).max())
        print(f"  op {n}: rel_l2={err:.3e}", flush=True)
        assert np.all(np.isfinite(got[d]))
        assert err <= TOL, (n, err)


@pytest.mark.parametrize("T,n_chain", [(3, 2), (5, 2), (3, 8), (5, 8)])
def test_prepared_odd_batches_on_pure_chains(T, n_chain):
    """Odd T on a chain in which every op is a stage of its own: the last pass holds one token, and
    the workspace that rb_workspace_bytes reports must be enough for it."""
    rng = synth.child_rng(3, 500 + 10 * T + n_chain)
    d = 4096
    layers = [random_layer(rng, 2, d, d, gain=100.0) for _ in range(n_chain)]
    x = synth.outlier_activations(rng, T, d)
    dev_layers = [to_device_layer(*l) for l in layers]
    bufs = [torch.zeros((T, d), dtype=torch.float16, device="cuda") for _ in range(n_chain + 1)]
    bufs[0].copy_(torch.from_numpy(x))
    op_list = [(n, n, n + 1) for n in range(n_chain)]
    print(f"pure chain of {n_chain} ops, T={T}", flush=True)
    stack = rb.Stack(dev_layers, op_list, bufs, T)
    stack.prepare()
    stack.run_prepared()
    torch.cuda.synchronize()
    assert stack.status() == rb.RB_OK, f"gave up: reason {stack.gave_up()}"
    stack.forget()
    got = [b.cpu().numpy() for b in bufs]
    for n in range(n_chain):
        ref = oracle.forward(*layers[n], got[n])
        err = float(oracle.relative_l2(got[n + 1].astype(np.float64), ref).max())
        assert np.all(np.isfinite(got[n + 1])) and err <= TOL, (n, err)
