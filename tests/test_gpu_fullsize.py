"""GPU parity at the full sizes of the paper's workloads (CaffeNet-shaped layers at batch 256, the
CIFAR-style stack at batch 128), in the launch configuration the bench times.

The direct-loop oracle needs minutes to hours for whole tensors at these sizes, so it evaluates
randomly sampled entries one by one (`*_at` routines) and, where a whole-tensor check is cheap
(pooling, ReLU, bias gradient, the update), the whole tensor.  Each stage of a chained stack is
compared with the oracle applied to the inputs that stage received on the GPU.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}
N_SAMPLES = 3000


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


def gpu(a, dtype=0):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == 1 else t


def host32(t):
    return t.detach().float().cpu().numpy()


def sample_err(got_tensor, ref_fn, rng, count=N_SAMPLES):
    """max |gpu - oracle| over sampled entries, normalised by the largest sampled |oracle| value."""
    flat = got_tensor.detach().reshape(-1)
    idx = np.unique(rng.integers(0, flat.numel(), size=count))
    got = flat[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)
    ref = ref_fn(idx)
    return np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30)


def oshape(L):
    return oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)


def check_layer(B, L, dtype, seed, x_dist="normal", dgrad=True):
    t = wl.layer_tensors(L, seed=seed, x_dist=x_dist, bf16=(dtype == 1))
    s = oshape(L)
    d = B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype)
    X, W, dY, bias = gpu(t["X"], dtype), gpu(t["W"], dtype), gpu(t["dY"], dtype), gpu(t["bias"])
    rng = np.random.default_rng(seed + 100)
    nbytes = max(B.conv_workspace_bytes(d, B.PASS_FORWARD), B.conv_workspace_bytes(d, B.PASS_BACKWARD_WEIGHTS))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Y = B.conv_forward(d, X, W, bias, workspace=ws)
    e = sample_err(Y, lambda i: oracle.conv_forward_at(s, t["X"], t["W"], t["bias"], i), rng)
    assert e <= TOL[dtype], ("forward", L.name, e)
    dW, db = B.conv_backward_weights(d.with_flags(B.FLAG_DHAT_CACHED), None, dY, workspace=ws)
    e = sample_err(dW, lambda i: oracle.conv_backward_weights_at(s, t["X"], t["dY"], i), rng, 300)
    assert e <= 1e-4, ("backward_weights", L.name, e)
    ref_db = oracle.bias_grad(s, t["dY"])
    assert np.max(np.abs(host32(db) - ref_db)) / np.max(np.abs(ref_db)) <= 1e-4
    del ws
    if dgrad:
        dX = B.conv_backward_data(d, dY, W)
        e = sample_err(dX, lambda i: oracle.conv_backward_data_at(s, t["dY"], t["W"], i), rng)
        assert e <= TOL[dtype], ("backward_data", L.name, e)
    torch.cuda.synchronize()


def test_caffenet_conv1_fp32_batch256(B):
    # forward, data gradient and model gradient of the 11x11 stride-4 layer on 256 images
    check_layer(B, wl.caffenet_stack(256)[0], 0, seed=1)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("which", [1, 2, 3, 4])
def test_caffenet_conv2_to_conv5_batch256(B, which, dtype):
    check_layer(B, wl.caffenet_stack(256)[which], dtype, seed=1 + which)


def test_cifar_layers_fp32_batch128(B):
    for i, L in enumerate(wl.cifar_stack(128)):
        check_layer(B, L, 0, seed=10 + i, x_dist="uniform")


def check_stack(B, layers, dtype, ceil_mode, x_dist, seed, skip_first_dgrad, lr=0.01, mu=0.9):
    from paper_1606_04487_amd.stack import ConvStack
    st = ConvStack(layers, dtype=dtype, ceil_mode=ceil_mode, skip_first_dgrad=skip_first_dgrad)
    data = wl.stack_tensors(layers, seed=seed, x_dist=x_dist, bf16=(dtype == 1), pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    X, dOut = gpu(data["X"], dtype), gpu(data["dY"], dtype)
    st.forward(X)
    st.backward(dOut)
    torch.cuda.synchronize()
    rng = np.random.default_rng(seed + 7)
    tol = TOL[dtype]
    g_in = dOut
    for i in reversed(range(len(layers))):
        L, s = layers[i], oshape(layers[i])
        Xi, Wi, bi = host32(st.X[i]), host32(st.Wc[i]), data["bias"][i]
        e = sample_err(st.Y[i], lambda idx: np.maximum(oracle.conv_forward_at(s, Xi, Wi, bi, idx), 0), rng)
        assert e <= tol, ("forward", L.name, e)
        Yg = host32(st.Y[i])
        if L.pool_after:
            Pref, Aref = oracle.maxpool_forward(Yg, 3, 2, ceil_mode)
            assert np.array_equal(host32(st.P[i]).astype(np.float64), Pref), ("pool", L.name)
            dYr = oracle.maxpool_backward(host32(g_in), Aref, L.Ho, L.Wo)
        else:
            dYr = host32(g_in).astype(np.float64)
        Gg = host32(st.dYc[i])
        # each pixel sums the gradients of the (at most four) windows it won: fp32 on the GPU, rounded once on store
        ref = oracle.relu_backward(Yg, np.ones_like(Yg)) * dYr
        tol_g = 1e-6 if dtype == 0 else tol
        assert np.max(np.abs(Gg - ref)) <= tol_g * max(np.max(np.abs(ref)), 1e-30), ("relu/pool backward", L.name)
        assert np.all(Gg[Yg <= 0] == 0)
        e = sample_err(st.dW[i], lambda idx: oracle.conv_backward_weights_at(s, Xi, Gg, idx), rng, 200)
        assert e <= 1e-4, ("backward_weights", L.name, e)
        ref_db = oracle.bias_grad(s, Gg)
        assert np.max(np.abs(host32(st.db[i]) - ref_db)) <= 1e-4 * max(np.max(np.abs(ref_db)), 1e-30)
        if st.dXl[i] is None:
            break
        e = sample_err(st.dXl[i], lambda idx: oracle.conv_backward_data_at(s, Gg, Wi, idx), rng)
        assert e <= tol, ("backward_data", L.name, e)
        g_in = st.dXl[i]
    # the update, whole tensors
    W0 = [host32(w) for w in st.W]
    b0 = [host32(b) for b in st.b]
    dW = [host32(g) for g in st.dW]
    db = [host32(g) for g in st.db]
    st.sgd_step(lr, mu)
    for i in range(len(layers)):
        W1, V1 = oracle.sgd_momentum(W0[i], np.zeros_like(W0[i]), dW[i], np.float32(lr), np.float32(mu), 0.0)
        b1, _ = oracle.sgd_momentum(b0[i], np.zeros_like(b0[i]), db[i], np.float32(lr), np.float32(mu), 0.0)
        assert np.max(np.abs(host32(st.W[i]) - W1)) <= 1e-6 * np.max(np.abs(W1))
        assert np.max(np.abs(host32(st.VW[i]) - V1)) <= 1e-6 * max(np.max(np.abs(V1)), 1e-30)
        assert np.max(np.abs(host32(st.b[i]) - b1)) <= 1e-6 * np.max(np.abs(b1))
        if dtype == 1:
            assert torch.equal(st.Wc[i], st.W[i].to(torch.bfloat16))
    del st
    torch.cuda.empty_cache()


def test_cifar_stack_fp32_batch128(B):
    check_stack(B, wl.cifar_stack(128), 0, True, "uniform", seed=1, skip_first_dgrad=False)


@pytest.mark.parametrize("dtype", [0, 1])
def test_caffenet_conv2_to_conv5_chained_batch256(B, dtype):
    layers = wl.caffenet_stack(256)[1:]
    check_stack(B, layers, dtype, False, "normal", seed=2, skip_first_dgrad=False)


@pytest.mark.parametrize("N", [1, 16, 64, 256])
def test_caffenet_full_stack_bf16_batch_sweep(B, N):
    # the configuration the bench times (N = 256), and the smaller batches of the sweep
    check_stack(B, wl.caffenet_stack(N), 1, False, "normal", seed=3, skip_first_dgrad=True)


def test_repeated_steps_stay_finite_and_in_distribution(B):
    # the bench's loop (forward, backward, momentum update on the same batch) at batch 16: thirty steps must
    # leave every tensor finite, every layer's output alive and the weights where they were drawn
    from paper_1606_04487_amd.stack import ConvStack
    N = 16
    layers = wl.caffenet_stack(N)
    st = ConvStack(layers, dtype=1, ceil_mode=False, skip_first_dgrad=True)
    data = wl.stack_tensors(layers, seed=1, bf16=True, pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    X = gpu(data["X"], 1)
    dOut = (torch.from_numpy(data["dY"]).cuda() * wl.step_upstream_scale(N)).to(torch.bfloat16)
    W0 = [w.clone() for w in st.W]
    first = None
    for step in range(30):
        st.step(X, dOut, 0.01, 0.9)
        if step == 0:
            first = st.tensor_health(W0)
    h = st.tensor_health(W0)
    assert h["finite"] and not ConvStack.health_is_degenerate(h), h
    assert all(0.3 < z < 0.7 for z in h["zero_fraction_Y"]), h      # ReLU of a zero-mean input: about half
    assert all(c <= 0.01 * 0.01 for c in h["max_abs_W_change"]), h  # under a hundredth of sigma after 30 steps
    assert all(c > 0 for c in h["max_abs_W_change"]), h             # but the update did move the weights
    for a, b in zip(first["max_abs_Y"], h["max_abs_Y"]):
        assert abs(a - b) <= 0.05 * a, (first, h)
    del st
    torch.cuda.empty_cache()
