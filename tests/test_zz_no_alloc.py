"""The forward entry point that allocates nothing (omni_conv_forward_static) against omni_conv_forward:
same kernels on the library's static device scratch instead of a caller's workspace, so the outputs must be
bit-identical.  Two calls in a row share the scratch, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


def run_pair(B, N, C, H, F, k, s, p, dtype, flags, seed):
    L = wl.ConvLayer("t", N, C, H, H, F, k, s, p)
    t = wl.layer_tensors(L, seed=seed, bf16=(dtype == 1))
    td = B.torch_dtype(dtype)
    X, W = (torch.from_numpy(t[n]).cuda().to(td) for n in ("X", "W"))
    bias = torch.from_numpy(t["bias"]).cuda()
    d = B.conv_desc(N, C, H, H, F, k, k, s, p, dtype, flags)
    assert B.conv_static_scratch_need(d) <= B.STATIC_SCRATCH_BYTES
    ref = B.conv_forward(d, X, W, bias)                       # the existing entry point, caller's workspace
    ho, wo = B.conv_output_dims(d)
    Y = torch.full((N, F, ho, wo), float("nan"), dtype=td, device="cuda")
    B.conv_forward_static(d, X, W, bias, Y)                   # through the C ABI, no workspace argument
    torch.cuda.synchronize()
    assert torch.isfinite(ref.float()).all()
    assert torch.equal(Y.view(torch.int16 if dtype == 1 else torch.int32),
                       ref.view(torch.int16 if dtype == 1 else torch.int32)), (N, C, H, F, k, s, p, dtype, flags)
    return X, W, bias, ref


def test_static_scratch_forward_matches_the_workspace_entry_point(B):
    # explicit path (lowering + GEMM in the scratch), fp32: the larger call first, then a smaller one that
    # finds the first call's D-hat and K-hat still lying in the scratch
    X, W, bias, ref = run_pair(B, 8, 3, 32, 32, 5, 1, 2, 0, B.FLAG_RELU, seed=1)
    run_pair(B, 3, 3, 19, 20, 3, 2, 1, 0, 0, seed=2)
    # the first layer again: nothing of the smaller call may leak into it
    d = B.conv_desc(8, 3, 32, 32, 32, 5, 5, 1, 2, 0, B.FLAG_RELU)
    Y = torch.empty_like(ref)
    B.conv_forward_static(d, X, W, bias, Y)
    torch.cuda.synchronize()
    assert torch.equal(Y, ref)


def test_static_scratch_forward_fused_and_bf16(B):
    # fused passes keep only their repacked weights in the scratch: a CaffeNet conv4-shaped layer at batch 4 (its reduction split, the partial sums in the scratch too),
    # then a smaller fused layer, then a small explicit bf16 layer and the stride-4 kernel
    run_pair(B, 4, 384, 13, 384, 3, 1, 1, 1, B.FLAG_FUSED | B.FLAG_RELU, seed=3)
    run_pair(B, 4, 32, 13, 64, 3, 1, 1, 1, B.FLAG_FUSED, seed=4)
    run_pair(B, 5, 7, 17, 24, 3, 1, 1, 1, 0, seed=5)
    run_pair(B, 2, 3, 67, 96, 11, 4, 0, 1, B.FLAG_FUSED, seed=6)


def test_static_scratch_refuses_what_does_not_fit(B):
    d = B.conv_desc(256, 96, 27, 27, 256, 5, 5, 1, 2, 1)        # explicit path at batch 256: 900 MB of D-hat
    assert B.conv_static_scratch_need(d) > B.STATIC_SCRATCH_BYTES
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    st = B.raw().omni_conv_forward_static(ctypes.byref(d), x.data_ptr(), x.data_ptr(), None, x.data_ptr(), None)
    assert st == -3
