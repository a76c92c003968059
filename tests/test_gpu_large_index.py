"""GPU parity beyond 32-bit indices: a batch whose lowered matrix has more than 2^31 elements (4.8 GB in bf16).

Lowering, col2im and the three passes are independent per image except for the model gradient's sum over the
batch, so images at the start, the middle and the end of the batch (whose columns of the lowered matrix lie
beyond element 2^31 in its last rows) are compared with the oracle applied to those images alone; the model
gradient is compared entry by entry on sampled entries, which the oracle sums over the whole batch.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu

N, C, H, F, K, P = 4096, 32, 27, 32, 5, 2
IMAGES = (0, 1, 2047, 2900, 4094, 4095)
TOL = 2e-2


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def data():
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2 ** 30:
        pytest.skip("needs 40 GB of free device memory")
    rng = np.random.default_rng(11)
    X = wl.to_bf16_values(rng.standard_normal((N, C, H, H), dtype=np.float32))
    W = wl.to_bf16_values((0.05 * rng.standard_normal((F, C, K, K))).astype(np.float32))
    bias = (0.05 * rng.standard_normal(F)).astype(np.float32)
    dY = wl.to_bf16_values(rng.standard_normal((N, F, H, H), dtype=np.float32))
    dev = {k: torch.from_numpy(v).cuda().to(torch.bfloat16) for k, v in (("X", X), ("W", W), ("dY", dY))}
    dev["bias"] = torch.from_numpy(bias).cuda()
    return {"X": X, "W": W, "bias": bias, "dY": dY, "dev": dev}


def one(s_n=1):
    return oracle.shape(s_n, C, H, H, F, K, K, 1, P)


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def test_lowered_matrix_has_more_than_2_31_elements():
    assert C * K * K * N * H * H > 2 ** 31 and C * K * K * N * H * H * 2 > 2 ** 32


def test_lower_and_col2im(B, data):
    d = B.conv_desc(N, C, H, H, F, K, K, 1, P, B.BF16)
    ld = B.conv_dhat_ld(d)
    Dhat = B.lower(d, data["dev"]["X"], ld=ld)
    hw = H * H
    for n in IMAGES:
        ref = oracle.lower(one(), data["X"][n:n + 1])
        got = Dhat[:, n * hw:(n + 1) * hw].float().cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), n
    assert not bool(torch.any(Dhat[:, N * hw:] != 0))
    dX = B.col2im(d, Dhat, ld=ld)
    for n in IMAGES:
        D1 = Dhat[:, n * hw:(n + 1) * hw].float().cpu().numpy()
        ref = oracle.col2im(one(), D1)
        got = dX[n:n + 1].float().cpu().numpy().astype(np.float64)
        assert rel_err(got, ref) <= 2.0 ** -8, n     # one rounding to bf16 of an fp32 sum of at most 25 terms
    del Dhat, dX
    torch.cuda.empty_cache()


@pytest.mark.parametrize("fused", [False, True])
def test_three_passes(B, data, fused):
    d = B.conv_desc(N, C, H, H, F, K, K, 1, P, B.BF16, B.FLAG_FUSED if fused else 0)
    dev = data["dev"]
    Y = B.conv_forward(d, dev["X"], dev["W"], dev["bias"])
    dX = B.conv_backward_data(d, dev["dY"], dev["W"])
    dW, db = B.conv_backward_weights(d, dev["X"], dev["dY"])
    torch.cuda.synchronize()
    for n in IMAGES:
        ref = oracle.conv_forward(one(), data["X"][n:n + 1], data["W"], data["bias"])
        assert rel_err(Y[n:n + 1].float().cpu().numpy(), ref) <= TOL, ("forward", n)
        ref = oracle.conv_backward_data(one(), data["dY"][n:n + 1], data["W"])
        assert rel_err(dX[n:n + 1].float().cpu().numpy(), ref) <= TOL, ("data gradient", n)
    rng = np.random.default_rng(12)
    idx = np.unique(rng.integers(0, F * C * K * K, size=96))
    ref = oracle.conv_backward_weights_at(one(N), data["X"], data["dY"], idx)
    got = dW.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy().astype(np.float64)
    full_scale = float(np.max(np.abs(dW.cpu().numpy())))
    assert float(np.max(np.abs(got - ref))) / full_scale <= TOL
    ref_b = data["dY"].astype(np.float64).sum(axis=(0, 2, 3))
    assert rel_err(db.cpu().numpy().astype(np.float64), ref_b) <= TOL
    del Y, dX, dW
    torch.cuda.empty_cache()
