#!/usr/bin/env python3
"""Benchmark of the residual-binary decode path on one MI355X.

A step is one pass of the whole hot path over one token: input scaling,
signed accumulation, row reduction, output scaling and path sum for all 224
matrices of the Llama-7B-shaped K=2 stack, in dependency order, through
``rb_stack_run`` (set-up that depends only on the frozen weights is done once
by ``rb_stack_prepare``, like packing).  Weights are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def build_stack(rb, synth, torch, which: str, T: int, seed: int = 20260205, K: int = 2):
    """Synthetic Llama-shaped stack resident on the GPU.

    Sign words are i.i.d. uniform bits drawn on the device directly in the
    native tile order (a permutation of i.i.d. bits is i.i.d.).  Scales follow
    what the paper's derivation gives for W ~ N(0, 0.02^2): nearly constant
    g_k h_k (0.0160 for path 1, 0.0097 for path 2) with 1% jitter, and a
    per-op constant folded into g so that every op's output has RMS ~1.
    """
    ops, widths = synth.llama_stack(which)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    layers, packed_bytes = [], 0
    for n, op in enumerate(ops):
        nbytes = rb.rb_native_bytes(K, op.out, op.inn)
        bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda", generator=gen)
        gh = [0.0160, 0.0097, 0.0058][:K]            # third path: the residual shrinks by the same factor again
        a = torch.tensor(gh, device="cuda").sqrt()[:, None]
        c = 1.0 / (op.inn * sum(v ** 2 for v in gh)) ** 0.5
        g = (a * c * (1 + 0.01 * torch.randn(K, op.out, device="cuda", generator=gen))).half()
        h = (a * (1 + 0.01 * torch.randn(K, op.inn, device="cuda", generator=gen))).half()
        layers.append(rb.Layer(bits, g, h, K, op.out, op.inn))
        packed_bytes += K * op.out * op.inn // 8
    bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    bufs[0].copy_(torch.randn(T, widths[0], device="cuda", generator=gen).half())
    op_list = [(n, op.src, op.dst) for n, op in enumerate(ops)]
    return ops, layers, bufs, op_list, packed_bytes


def build_block_stack(rb, synth, torch, which: str, T: int, seed: int = 20260206, in_place: bool = True):
    """The same synthetic layers as build_stack with what sits between them in a decoder block
    (normalised q/k/v and gate/up inputs, silu(gate) * up, residual additions; attention left out),
    the residual stream kept in buffer 0 (`in_place`; otherwise every op writes a buffer of its own)."""
    ops, shapes, widths, norms = synth.llama_block_stack(which, synth.LLAMA_SHAPES[which][2], in_place=in_place)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    layers, packed_bytes = [], 0
    gh = [0.0160, 0.0097]
    a = torch.tensor(gh, device="cuda").sqrt()[:, None]
    for name, out, inn in shapes:
        bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (rb.rb_native_bytes(2, out, inn) // 4,), dtype=torch.int32,
                             device="cuda", generator=gen)
        c = 1.0 / (inn * sum(v ** 2 for v in gh)) ** 0.5 * (2.0 if name.endswith("down") else 1.0)
        g = (a * c * (1 + 0.01 * torch.randn(2, out, device="cuda", generator=gen))).half()
        h = (a * (1 + 0.01 * torch.randn(2, inn, device="cuda", generator=gen))).half()
        layers.append(rb.Layer(bits, g, h, 2, out, inn))
        packed_bytes += 2 * out * inn // 8
    norm_w = [(1 + 0.1 * torch.randn(w, device="cuda", generator=gen)).half() for w in norms]
    bufs = [torch.zeros((T, w), dtype=torch.float16, device="cuda") for w in widths]
    x0 = torch.randn(T, widths[0], device="cuda", generator=gen).half()
    op_list = [(o.layer, o.src, o.dst, o.norm, o.epilogue, o.aux) for o in ops]
    return ops, layers, norm_w, bufs, x0, op_list, packed_bytes


def time_steps(torch, fn, steps: int, warmup: int):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]      # ms, on the launch stream
    return wall, per


def cpu_baseline(synth, packed_bytes_total: int):
    """The oracle as it stands, on the host cores, on one of the 32 blocks."""
    import numpy as np
    import oracle
    ops, widths = synth.llama_stack("7b", n_layers=1)
    rng = synth.child_rng(2, 99)
    mats = []
    for op in ops:
        mats.append((synth.uniform_signs(rng, 2, op.out, op.inn),
                     synth.halfnormal_scales(rng, 2, op.out), synth.halfnormal_scales(rng, 2, op.inn),
                     synth.gaussian_activations(rng, 1, op.inn)))
    sample_bytes = sum(2 * op.out * op.inn // 8 for op in ops)
    oracle.forward(*mats[0])                                     # load the library, warm the pages
    reps, t0 = 0, time.perf_counter()
    while reps < 2 or time.perf_counter() - t0 < 10.0:
        for m in mats:
            oracle.forward(*m)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": sample_bytes / dt / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"1 of 32 blocks (7 matrices, {sample_bytes} packed bytes), forward only, "
                      f"{reps} repetitions, {dt:.3f} s each",
            "tokens_per_s_extrapolated": 1.0 / (dt * packed_bytes_total / sample_bytes)}


def prefill_figures(rb, torch):
    """Prefill GEMM (configs[4]): T = 2048 tokens, 70B-shaped MLP matrices, bf16 activations."""
    prefill = {}
    Tp = 2048
    for (o, i, Kp) in ((28672, 8192, 2), (8192, 28672, 2), (8192, 28672, 3)):
        nb = rb.rb_native_bytes(Kp, o, i)
        bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (nb // 4,), dtype=torch.int32, device="cuda")
        gg = (torch.randn(Kp, o, device="cuda").abs() * 0.02).half()
        hh = (torch.randn(Kp, i, device="cuda").abs() * 0.02).half()
        Lp = rb.Layer(bits, gg, hh, Kp, o, i)
        Xp = torch.randn((Tp, i), device="cuda").to(torch.bfloat16)
        Yp = torch.empty((Tp, o), dtype=torch.float16, device="cuda")
        wsp = rb.binding._workspace([Lp], Tp, Xp.device)
        _, per_p = time_steps(torch, lambda: rb.rb_linear_gemm(Lp, Xp, Y=Yp, workspace=wsp), 8, 2)
        msp = sum(per_p) / len(per_p)
        # The kernel contracts once, with the effective weight built in registers (Alg. 2's dense
        # form Y = W_hat X): 2 out in T flops on the matrix units, whatever K.  By the layer's
        # definition (K contractions of +-1 matrices) the same call is K times that; both are given.
        flops = 2.0 * o * i * Tp
        prefill[f"{o}x{i}" + ("" if Kp == 2 else f"_K{Kp}")] = {
            "ms": msp, "TFLOPs": flops / msp / 1e9, "frac_of_fp16_mfma_peak": flops / msp / 1e9 / 2500.0,
            "flops_counted": "2 out in T: the matrix instructions issued (one contraction)",
            "TFLOPs_by_definition": Kp * flops / msp / 1e9,
            "definition": "2 K out in T: K contractions of +-1 matrices, the form the two-contraction kernel ran (1.92-2.02 ms)"}
        del bits, Lp, Xp, Yp, wsp
    return prefill


def training_figures(rb, torch):
    """Training-side kernels (Alg. 2) and the initialisation (Alg. 1) on one 4096 x 11008 layer."""
    out = {}
    # training-side kernels (Alg. 2): coupled derivation of the cores and the scale gradients
    # of one 4096 x 11008 layer; both stream an fp32 matrix, so the figure is HBM bytes per second
    o_t, i_t = 4096, 11008
    Wt = torch.randn((o_t, i_t), device="cuda") * 0.02
    gt = (torch.randn(2, o_t, device="cuda").abs() * 0.1).half()
    ht = (torch.randn(2, i_t, device="cuda").abs() * 0.1).half()
    _, per_c = time_steps(torch, lambda: rb.rb_couple(Wt, gt, ht), 10, 3)
    pk, _, _ = rb.rb_couple(Wt, gt, ht)
    ms_c = sum(per_c) / len(per_c)
    bytes_c = 4 * o_t * i_t + 2 * (2 * o_t * i_t // 8)         # W read, canonical and native words written
    _, per_g = time_steps(torch, lambda: rb.rb_scale_grads(Wt, pk, gt, ht), 10, 3)
    ms_g = sum(per_g) / len(per_g)
    bytes_g = 4 * o_t * i_t + 2 * o_t * i_t // 8               # G and the packed cores, read once for both gradients
    out["training_side_4096x11008"] = {
        "rb_couple": {"ms": ms_c, "GBps": bytes_c / (ms_c * 1e-3) / 1e9,
                      "pct_of_hbm_peak": 100.0 * bytes_c / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "rb_scale_grads": {"ms": ms_g, "GBps": bytes_g / (ms_g * 1e-3) / 1e9,
                           "pct_of_hbm_peak": 100.0 * bytes_g / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBPS}}
    # initialisation (Alg. 1): Iterative Residual SVID of the same layer on the device, fp64;
    # wall clock of the call (it follows the power iteration's stopping rule from the host)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, _, _, err_i = rb.rb_derive_iterative(Wt, 2, 5)
    torch.cuda.synchronize()
    s_i = time.perf_counter() - t0
    err_i = err_i.cpu().numpy()
    out["initialisation_4096x11008"] = {
        "rb_derive_iterative": {"K": 2, "T_max": 5, "seconds": s_i, "seconds_per_sweep": s_i / 5,
                                "error_after_greedy_over_norm": float(err_i[0, 1] / Wt.double().norm().item()),
                                "error_after_5_sweeps_over_norm": float(err_i[4, 1] / Wt.double().norm().item())}}
    del Wt, pk
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-extras", action="store_true", help="skip comparators and the CPU baseline")
    ap.add_argument("--prefill-only", action="store_true",
                    help="only the prefill GEMM figures (for profiling that kernel)")
    ap.add_argument("--batch-only", type=int, default=0, metavar="T",
                    help="only the dependent 7B-shaped chain at T tokens (8..16) on the small-batch kernel (for profiling it)")
    ap.add_argument("--block-only", type=int, default=0, metavar="T",
                    help="only the 7B-shaped decoder-block stack at T tokens (1..4) on the fused kernel (for profiling it)")
    ap.add_argument("--train-only", action="store_true",
                    help="only the training-side kernels and the initialisation (for profiling them)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) for counter calibration")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        return 2

    import torch
    import synth
    import paper_2602_05367_amd as rb
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.prefill_only:
        print(json.dumps({"prefill_gemm_T2048": prefill_figures(rb, torch)}))
        return 0

    if args.train_only:
        print(json.dumps(training_figures(rb, torch)))
        return 0

    if args.batch_only:
        Tb = args.batch_only
        ops_b, layers_b, bufs_b, op_list_b, packed_b = build_stack(rb, synth, torch, "7b", Tb)
        st_b = rb.Stack(layers_b, op_list_b, bufs_b, Tb)
        st_b.prepare()
        _, per_b = time_steps(torch, st_b.run_prepared, args.steps, args.warmup)
        assert rb.rb_last_path() == rb.RB_PATH_BATCH and st_b.status() == rb.RB_OK
        ms_b = sum(per_b) / len(per_b)
        print(json.dumps({"small_batch_chain": {"tokens": Tb, "ms_per_pass": ms_b, "tokens_per_s": Tb / (ms_b * 1e-3),
                                                "GBps": packed_b / (ms_b * 1e-3) / 1e9}}))
        return 0

    if args.block_only:
        Tb = args.block_only
        bops, blayers, bnorms, bbufs, bx0, bop_list, bpacked = build_block_stack(rb, synth, torch, "7b", Tb)
        block = rb.Block(blayers, bnorms, 1e-5, bop_list, bbufs, Tb)
        block.prepare()

        def fused_step():
            bbufs[0].copy_(bx0)
            block.run_prepared()
        _, per_b = time_steps(torch, fused_step, args.steps, args.warmup)
        assert rb.rb_last_path() == rb.RB_PATH_MX and block.status() == rb.RB_OK
        ms_b = sum(per_b) / len(per_b)
        print(json.dumps({"decoder_block_stack_7b": {"tokens": Tb, "ms_per_pass": ms_b, "tokens_per_s": Tb / (ms_b * 1e-3),
                                                     "GBps": bpacked / (ms_b * 1e-3) / 1e9}}))
        return 0

    T = 1
    ops, layers, bufs, op_list, packed_bytes = build_stack(rb, synth, torch, "7b", T)
    stack = rb.Stack(layers, op_list, bufs, T)
    stack.prepare()
    wall, per = time_steps(torch, stack.run_prepared, args.steps, args.warmup)
    assert rb.rb_last_path() == rb.RB_PATH_MX
    assert stack.status() == rb.RB_OK, "a run of the timed stack gave up a hand-over wait"
    ms = sum(per) / len(per)
    ms_min = min(per)
    y = bufs[ops[-1].dst].float()
    assert torch.isfinite(y).all() and float(y.abs().max()) > 0

    result = {
        "metric": "packed-weight HBM GB/s, decode, Llama-7B-shaped K=2 stack (224 residual-binary GEMVs in "
                  "dependency order, linear layers only)",
        "value": packed_bytes / (ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp16 in/out, fp4 signs x 4-term bf8 inputs on MFMA, fp32 accumulate", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-7B-shaped decode stack, batch 1, K=2, 32 blocks x "
                               "(q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008); i.i.d. sign bits, "
                               "scales as the paper's derivation gives for Gaussian weights",
                   "tokens": T, "packed_bytes": packed_bytes, "workspace_bytes": stack.ws_bytes,
                   "entry_point": "rb_stack_run"},
        "tokens_per_s": T / (ms * 1e-3),
        "pct_of_hbm_peak": 100.0 * packed_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "us_per_layer": ms * 1e3 / len(ops),
        "ms_per_step_min": ms_min,
        "ms_per_step_median": sorted(per)[len(per) // 2],
        "wall_ms_per_step": wall * 1e3 / args.steps,
        # input tiles (of 1,581,056 per token) that were requested before their producer had written
        # them and had to be waited for: what the pacing of the hand-over costs
        "tiles_waited_per_step": stack.waited() / float(args.steps + args.warmup),
    }
    # HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, scaled
    # by what the same counters read for a plain copy of known size)
    traffic = None
    pmc = os.path.join(ROOT, "profiles", "stack_kernel_7b_T1_pmc.txt")
    if os.path.exists(pmc):
        import re
        m = re.search(r"hbm_bytes_per_launch\s*:\s*(\d+)", open(pmc).read())
        traffic = int(m.group(1)) if m else None
    result["roofline"] = {
        "bound": "hbm", "kernel": "rb::mx::stack_kernel",
        "achieved": packed_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": packed_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "traffic": traffic,
        "traffic_source": "profiles/stack_kernel_7b_T1_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                          "scaled by a plain copy of known size; counters cannot be read from inside this process)",
        "note": "one launch per step; duration = HIP events around rb_stack_run on its stream "
                "(includes the ~6 us kernel that expands the stack input and marks inputs not yet written)",
    }

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_extras:
        # the same 224 matrices without data dependencies: every op reads the stack input or a
        # buffer nobody writes, so no cross-CU hand-over; this is the streaming rate of the kernel
        free_bufs = [torch.randn(T, w, device="cuda").half() for w in (4096, 11008)]
        outs = [torch.zeros((T, op.out), dtype=torch.float16, device="cuda") for op in ops]
        fb = free_bufs + outs
        free_ops = [(n, 0 if op.inn == 4096 else 1, 2 + n) for n, op in enumerate(ops)]
        free = rb.Stack(layers, free_ops, fb, T)
        free.prepare()
        _, per_f = time_steps(torch, free.run_prepared, max(20, args.steps // 4), 5)
        assert free.status() == rb.RB_OK
        ms_f = sum(per_f) / len(per_f)
        result["independent_ops"] = {"ms_per_step": ms_f, "GBps": packed_bytes / (ms_f * 1e-3) / 1e9,
                                     "pct_of_hbm_peak": 100.0 * packed_bytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        free.forget()
        # single calls (rb_linear_gemv) on the three 7B shapes: cold = rotating over distinct weight
        # copies (more than the 256 MB cache holds), warm = the same matrix again and again
        single = {}
        for (o, i) in ((4096, 4096), (11008, 4096), (4096, 11008)):
            nb = rb.rb_native_bytes(2, o, i)
            copies = max(80, (1 << 30) // nb)
            pool = torch.randint(-2 ** 31, 2 ** 31 - 1, (copies, nb // 4), dtype=torch.int32, device="cuda")
            gg = (torch.randn(2, o, device="cuda").abs() * 0.02).half()
            hh = (torch.randn(2, i, device="cuda").abs() * 0.02).half()
            Ls = [rb.Layer(pool[c], gg, hh, 2, o, i) for c in range(copies)]
            xs = torch.randn(1, i, device="cuda").half()
            ys = torch.empty((1, o), dtype=torch.float16, device="cuda")
            wss = rb.binding._workspace([Ls[0]], 1, xs.device)
            k = [0]

            def cold(Ls=Ls, xs=xs, ys=ys, wss=wss, k=k, copies=copies):
                rb.rb_linear_gemm(Ls[k[0] % copies], xs, Y=ys, workspace=wss)
                k[0] += 1
            _, per_c = time_steps(torch, cold, 160, 16)
            _, per_w = time_steps(torch, lambda: rb.rb_linear_gemm(Ls[0], xs, Y=ys, workspace=wss), 50, 10)
            pb = 2 * o * i // 8
            med_c, med_w = sorted(per_c)[len(per_c) // 2], sorted(per_w)[len(per_w) // 2]
            single[f"{o}x{i}"] = {"cold_us_median": med_c * 1e3, "cold_us_min": min(per_c) * 1e3,
                                  "cold_GBps": pb / (med_c * 1e-3) / 1e9,
                                  "warm_us_median": med_w * 1e3, "warm_GBps_cache_resident": pb / (med_w * 1e-3) / 1e9}
            del pool, Ls, wss
        result["single_call_gemv"] = single
        # the 13B-shaped stack (configs[3]): 40 blocks x (4 x 5120^2, 2 x 13824x5120, 5120x13824)
        ops13, layers13, bufs13, op_list13, packed13 = build_stack(rb, synth, torch, "13b", T)
        stack13 = rb.Stack(layers13, op_list13, bufs13, T)
        stack13.prepare()
        _, per13 = time_steps(torch, stack13.run_prepared, 30, 5)
        assert stack13.status() == rb.RB_OK
        ms13 = sum(per13) / len(per13)
        result["stack_13b"] = {"ms_per_token": ms13, "tokens_per_s": 1.0 / (ms13 * 1e-3), "packed_bytes": packed13,
                               "GBps": packed13 / (ms13 * 1e-3) / 1e9,
                               "pct_of_hbm_peak": 100.0 * packed13 / (ms13 * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        stack13.forget()
        del ops13, layers13, bufs13, stack13
        # two tokens per pass through the same 7B-shaped chain (both tokens share every MFMA)
        ops2, layers2, bufs2, op_list2, packed2 = build_stack(rb, synth, torch, "7b", 2)
        stack2 = rb.Stack(layers2, op_list2, bufs2, 2)
        stack2.prepare()
        _, per2 = time_steps(torch, stack2.run_prepared, 30, 5)
        assert stack2.status() == rb.RB_OK
        ms2 = sum(per2) / len(per2)
        result["stack_7b_two_tokens"] = {"ms_per_pass": ms2, "tokens_per_s": 2.0 / (ms2 * 1e-3),
                                         "GBps": packed2 / (ms2 * 1e-3) / 1e9,
                                         "tiles_waited_per_pass": stack2.waited() / 35.0}
        stack2.forget()
        del ops2, layers2, bufs2, stack2
        # three paths (the paper's 3-bit variant), the whole 7B-shaped chain: one token on the fused
        # decode kernel (one launch), eight on the small-batch kernel (one launch per group of independent ops)
        three = {}
        for T3 in (1, 8):
            ops3, layers3, bufs3, op_list3, packed3 = build_stack(rb, synth, torch, "7b", T3, K=3)
            stack3 = rb.Stack(layers3, op_list3, bufs3, T3)
            stack3.prepare()
            _, per3 = time_steps(torch, stack3.run_prepared, 20, 3)
            assert rb.rb_last_path() == (rb.RB_PATH_MX if T3 == 1 else rb.RB_PATH_BATCH) and stack3.status() == rb.RB_OK
            ms3 = sum(per3) / len(per3)
            three[f"T{T3}"] = {"ms_per_pass": ms3, "tokens_per_s": T3 / (ms3 * 1e-3), "packed_bytes": packed3,
                               "GBps": packed3 / (ms3 * 1e-3) / 1e9,
                               "pct_of_hbm_peak": 100.0 * packed3 / (ms3 * 1e-3) / 1e9 / HBM_PEAK_GBPS}
            stack3.forget()
            del ops3, layers3, bufs3, stack3
        result["three_path_stack_7b"] = three
        # whole decoder blocks in the same single launch: RMS normalisation in front of q/k/v and
        # gate/up, silu(gate) * up, both residual additions, all in the kernel's finishing step;
        # against the same block run op by op (a launch per layer and per elementwise operation)
        blocks = {}
        for Tb in (1, 4):
            bops, blayers, bnorms, bbufs, bx0, bop_list, bpacked = build_block_stack(rb, synth, torch, "7b", Tb)
            block = rb.Block(blayers, bnorms, 1e-5, bop_list, bbufs, Tb)
            block.prepare()

            def fused_step():
                bbufs[0].copy_(bx0)          # the residual stream lives in buffer 0: a fresh token every pass
                block.run_prepared()
            _, per_b = time_steps(torch, fused_step, 20, 3)
            assert rb.rb_last_path() == rb.RB_PATH_MX and block.status() == rb.RB_OK
            ms_b = sum(per_b) / len(per_b)
            blocks[f"T{Tb}"] = {"ms_per_pass": ms_b, "tokens_per_s": Tb / (ms_b * 1e-3), "GBps": bpacked / (ms_b * 1e-3) / 1e9,
                                "pct_of_hbm_peak": 100.0 * bpacked / (ms_b * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                "ops": len(bop_list), "matrices": len(blayers), "launches_per_pass": 1,
                                "entry_point": "rb_block_prepare + rb_stack_run"}
            if Tb == 1:
                def op_by_op():
                    x = bx0.clone()
                    for l in range(len(blayers) // 7):
                        L = blayers[7 * l: 7 * l + 7]
                        n1 = rb.rb_rmsnorm(x, bnorms[2 * l], 1e-5)
                        rb.rb_linear_gemm(L[0], n1); rb.rb_linear_gemm(L[1], n1)
                        v = rb.rb_linear_gemm(L[2], n1)
                        x = rb.rb_add(rb.rb_linear_gemm(L[3], v), x)
                        n2 = rb.rb_rmsnorm(x, bnorms[2 * l + 1], 1e-5)
                        act = rb.rb_silu_mul(rb.rb_linear_gemm(L[4], n2), rb.rb_linear_gemm(L[5], n2))
                        x = rb.rb_add(rb.rb_linear_gemm(L[6], act), x)
                _, per_u = time_steps(torch, op_by_op, 5, 2)
                blocks["T1"]["op_by_op_ms"] = sum(per_u) / len(per_u)
                blocks["T1"]["op_by_op_launches"] = 12 * (len(blayers) // 7)
            block.forget()
            del bops, blayers, bnorms, bbufs, block
        result["decoder_block_stack_7b"] = blocks
        # one-call form (set-up inside the call)
        _, per_o = time_steps(torch, stack.run, 20, 3)
        ms_o = sum(per_o) / len(per_o)
        result["rb_layer_stack_ms"] = ms_o
        result["roofline"]["rb_layer_stack"] = {"ms_per_step": ms_o, "achieved": packed_bytes / (ms_o * 1e-3) / 1e9,
                                                "frac": packed_bytes / (ms_o * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                                "note": "the same step through the one-call entry point: plan set-up inside the timed call"}
        # read-bandwidth ceiling of this device
        big = layers[4].bits
        blob = torch.empty(packed_bytes // 4, dtype=torch.int32, device="cuda")
        _, per_r = time_steps(torch, lambda: rb.rb_stream_read(blob), 20, 3)
        result["stream_read_GBps"] = packed_bytes / (min(per_r) * 1e-3) / 1e9
        del blob, big
        # hand-written dense fp16 GEMV on the same shapes (the paper's full-precision row)
        dense = {}
        for (o, i) in {(op.out, op.inn) for op in ops}:
            W = torch.empty((8, o, i), dtype=torch.float16, device="cuda").normal_(0, 0.02)   # > L2 + MALL
            x = torch.randn(i, device="cuda").half()
            yb = torch.empty(o, dtype=torch.float16, device="cuda")
            k = [0]

            def run(W=W, x=x, yb=yb, k=k):
                rb.rb_dense_gemv_f16(W[k[0] % 8], x, yb)
                k[0] += 1
            _, per_d = time_steps(torch, run, 32, 8)
            dense[f"{o}x{i}"] = sum(per_d) / len(per_d) * 1e3
            del W
        per_tok_us = 32 * (4 * dense["4096x4096"] + 2 * dense["11008x4096"] + dense["4096x11008"])
        result["dense_fp16_gemv"] = {"us_per_matrix": dense, "tokens_per_s": 1e6 / per_tok_us,
                                     "GBps": 2 * 8 * packed_bytes / 2 / (per_tok_us * 1e-6) / 1e9}
        result["speedup_vs_dense_fp16"] = result["tokens_per_s"] / result["dense_fp16_gemv"]["tokens_per_s"]
        result["paper_context"] = "RTX 4090: 291.88 tok/s = 4.49x FP16, whole Llama2-7B model (inference table)"
        result["prefill_gemm_T2048"] = prefill_figures(rb, torch)
        # small decode batches (configs[2]): the 7B-shaped stack, every op on its own input buffer.
        # 2 and 4 tokens: the fused decode kernel, one launch (four tokens are two pairs that share the
        # expanded signs).  8 and 16 tokens: the small-batch kernel,
        # one pass over the weights, one launch per group of independent ops.
        skinny = {}
        for Ts in (2, 4, 8, 16):
            fbs = [torch.randn(Ts, w, device="cuda").half() for w in (4096, 11008)]
            outs_s = [torch.zeros((Ts, op.out), dtype=torch.float16, device="cuda") for op in ops]
            st_s = rb.Stack(layers, [(n, 0 if op.inn == 4096 else 1, 2 + n) for n, op in enumerate(ops)], fbs + outs_s, Ts)
            st_s.prepare()
            _, per_s = time_steps(torch, st_s.run_prepared, 8, 2)
            assert st_s.status() == rb.RB_OK
            path = rb.rb_last_path()
            st_s.forget()
            ms_s = sum(per_s) / len(per_s)
            skinny[f"T{Ts}"] = {
                "ms_per_pass": ms_s, "tokens_per_s": Ts / (ms_s * 1e-3), "GBps": packed_bytes / (ms_s * 1e-3) / 1e9,
                "passes_over_the_weights": 1 if (Ts <= 4 or path == rb.RB_PATH_BATCH) else (Ts + 3) // 4,
                "kernel": "small-batch kernel" if path == rb.RB_PATH_BATCH else "fused decode kernel",
                "entry_point": "rb_stack_run"}
            del fbs, outs_s, st_s
        # the dependent 7B-shaped chain at 8 and 16 tokens (the small-batch kernel)
        for Ts in (8, 16):
            ops_b, layers_b, bufs_b, op_list_b, _ = build_stack(rb, synth, torch, "7b", Ts)
            st_b = rb.Stack(layers_b, op_list_b, bufs_b, Ts)
            st_b.prepare()
            _, per_b = time_steps(torch, st_b.run_prepared, 8, 2)
            assert rb.rb_last_path() == rb.RB_PATH_BATCH and st_b.status() == rb.RB_OK
            ms_b = sum(per_b) / len(per_b)
            skinny[f"T{Ts}_dependent_chain"] = {"ms_per_pass": ms_b, "tokens_per_s": Ts / (ms_b * 1e-3),
                                                "GBps": packed_bytes / (ms_b * 1e-3) / 1e9, "passes_over_the_weights": 1}
            st_b.forget()
            del ops_b, layers_b, bufs_b, st_b
        result["small_batch_stack"] = skinny
        result.update(training_figures(rb, torch))
        result["cpu_baseline"] = cpu_baseline(synth, packed_bytes)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
