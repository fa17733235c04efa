"""rb_linear_gemm_noalloc (scratch memory inside the library, nothing allocated) against
rb_linear_gemm (scratch memory from the caller) and the oracle: two calls in a row, the second on a
smaller input, so that what the first call left in the shared scratch array must not matter."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2602_05367_amd as rb
from helpers import TOL, random_layer, to_device_layer, max_rel_l2

pytestmark = pytest.mark.gpu


def test_noalloc_matches_workspace_variant_twice_second_call_smaller():
    rng = synth.child_rng(7, 0)
    big = random_layer(rng, 2, 528, 4096)
    small = random_layer(rng, 2, 272, 1024 + 32)
    Lb, Ls = to_device_layer(*big), to_device_layer(*small)
    Xb = synth.outlier_activations(rng, 16, 4096)
    Xs = synth.outlier_activations(rng, 5, 1024 + 32)
    for label, L, host, X in (("first call: 528x4096, T=16", Lb, big, Xb),
                              ("second call, smaller: 272x1056, T=5", Ls, small, Xs)):
        Xd = torch.from_numpy(X).cuda()
        want = rb.rb_linear_gemm(L, Xd)
        want_path = rb.rb_last_path()
        Y = torch.full((X.shape[0], L.out), float("nan"), dtype=torch.float16, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        print(label, flush=True)
        rb.rb_linear_gemm_noalloc(L, Xd, Y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert rb.rb_last_path() == want_path == rb.RB_PATH_GEMM      # the kernels that use scratch memory
        assert torch.equal(Y, want)
        assert max_rel_l2(Y, oracle.forward(*host, X)) <= TOL


def test_noalloc_three_paths_at_few_tokens():
    """Three-path layers: from six tokens on the one-contraction kernel on the library's scratch
    memory (the variant with a workspace may take the small-batch kernel instead: same result to
    the tolerance); below, and where that kernel's scratch would not fit, the generic kernel, which
    needs none."""
    rng = synth.child_rng(7, 2)
    host = random_layer(rng, 3, 272, 1056)
    L = to_device_layer(*host)
    for T, path in ((20, rb.RB_PATH_GEMM), (8, rb.RB_PATH_GEMM), (4, rb.RB_PATH_SIGNADD)):
        X = synth.outlier_activations(rng, T, 1056)
        Xd = torch.from_numpy(X).cuda()
        Y = torch.full((T, 272), float("nan"), dtype=torch.float16, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        print(f"three paths, T={T}", flush=True)
        rb.rb_linear_gemm_noalloc(L, Xd, Y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before and rb.rb_last_path() == path
        assert max_rel_l2(Y, oracle.forward(*host, X)) <= TOL
        if T == 20:
            assert torch.equal(Y, rb.rb_linear_gemm(L, Xd))          # the same kernel on the caller's workspace
    wide = random_layer(rng, 3, 16, 65536)                           # 256 x 65536 fp16 of scratch: more than the library holds
    Lw = to_device_layer(*wide)
    X = synth.gaussian_activations(rng, 8, 65536)
    Y = torch.full((8, 16), float("nan"), dtype=torch.float16, device="cuda")
    print("three paths, 65536 columns, T=8", flush=True)
    rb.rb_linear_gemm_noalloc(Lw, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    assert rb.rb_last_path() == rb.RB_PATH_SIGNADD
    assert max_rel_l2(Y, oracle.forward(*wide, X)) <= TOL


def test_noalloc_rejects_what_does_not_fit_and_bad_arguments():
    assert rb.rb_noalloc_scratch_bytes() == 32 << 20
    rng = synth.child_rng(7, 1)
    L = to_device_layer(*random_layer(rng, 2, 64, 8192))
    T = 2048                                             # 2 x 2048 x 8192 fp16 of scaled input: 64 MiB
    X = torch.zeros((T, 8192), dtype=torch.float16, device="cuda")
    Y = torch.zeros((T, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(rb.RabitError) as e:
        rb.rb_linear_gemm_noalloc(L, X, Y)
    assert e.value.code == rb.RB_ERR_WORKSPACE
    s = L.struct()
    assert rb.lib.rb_linear_gemm_noalloc(None, X.data_ptr(), Y.data_ptr(), 1, rb.RB_F16, rb.RB_F16, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_linear_gemm_noalloc(s, X.data_ptr(), None, 1, rb.RB_F16, rb.RB_F16, None) == rb.RB_ERR_NULL
    assert rb.lib.rb_linear_gemm_noalloc(s, X.data_ptr(), Y.data_ptr(), 0, rb.RB_F16, rb.RB_F16, None) == rb.RB_ERR_SHAPE
    assert rb.lib.rb_linear_gemm_noalloc(s, X.data_ptr(), Y.data_ptr(), 4, 7, rb.RB_F16, None) == rb.RB_ERR_UNSUPPORTED
