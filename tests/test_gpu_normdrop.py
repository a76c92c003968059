"""GPU parity of the normalisation and dropout layers (App. C, "Data Parallelism in non-GEMM Kernels")
against the CPU oracle, element by element.  Dropout's keep-mask is integer work (a counter-based generator
and a threshold) and must agree bit for bit; the kept values and the normalisation are floating point."""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


def gpu(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == 1 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


# (N, C, H, W, size, alpha, beta, k): CaffeNet's two normalisation layers at a reduced batch, ragged shapes,
# windows wider than the channel count, one channel, a large alpha that makes the scale matter
LRN_SHAPES = [
    (8, 96, 27, 27, 5, 1e-4, 0.75, 1.0), (8, 256, 13, 13, 5, 1e-4, 0.75, 1.0),
    (3, 7, 5, 9, 5, 0.5, 0.75, 1.0), (2, 3, 4, 4, 7, 1.0, 0.5, 2.0), (5, 1, 3, 3, 3, 0.3, 0.75, 1.0),
    (1, 33, 1, 1, 9, 2.0, 1.0, 0.5), (2, 16, 17, 3, 1, 0.7, 0.75, 1.0), (300, 4, 1, 2, 3, 0.1, 0.75, 1.0),
]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("N,C,H,W,size,alpha,beta,k", LRN_SHAPES)
def test_lrn_forward_and_backward(B, N, C, H, W, size, alpha, beta, k, dtype):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32) * 2.0
    g = rng.standard_normal((N, C, H, W)).astype(np.float32)
    if dtype == 1:
        x, g = wl.to_bf16_values(x), wl.to_bf16_values(g)
    xg, gg = gpu(x, dtype), gpu(g, dtype)
    y, scale = B.lrn_forward(xg, size, alpha, beta, k)
    dx = B.lrn_backward(xg, gg, scale, size, alpha, beta, k)
    y_only, none = B.lrn_forward(xg, size, alpha, beta, k, want_scale=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(y_only, y)
    # float32 parameters reach the kernel; hand the oracle the same values
    a32, b32, k32 = float(np.float32(alpha)), float(np.float32(beta)), float(np.float32(k))
    ref_y = oracle.lrn_forward(x, size, a32, b32, k32)
    ref_dx = oracle.lrn_backward(x, g, size, a32, b32, k32)
    x64 = x.astype(np.float64)
    ref_s = ref_y * 0 + k32
    for c in range(C):
        lo, hi = max(0, c - size // 2), min(C, c + size // 2 + 1)
        ref_s[:, c] = k32 + a32 / size * np.sum(x64[:, lo:hi] ** 2, axis=1)     # closed form of the window sum
    assert np.all(np.abs(host(scale) - ref_s) <= 2e-6 * np.abs(ref_s))
    tol = 2e-5 if dtype == 0 else 2.0 ** -8          # fp32 pow and a few flops; bf16: one rounding on store
    assert np.all(np.abs(host(y) - ref_y) <= tol * np.abs(ref_y) + 1e-30)
    # the gradient is a difference of two terms: bound the error by the terms' magnitudes, not by the result
    own = np.abs(g.astype(np.float64)) * ref_s ** -b32
    mag = own + np.abs(ref_dx - g.astype(np.float64) * ref_s ** -b32)
    assert np.all(np.abs(host(dx) - ref_dx) <= tol * mag + 1e-30)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("count,p,seed,stream_id", [(256 * 4096, 0.5, 1, 0), (1000003, 0.5, 7, 2), (7, 0.25, 3, 1), (8, 0.9, 2 ** 40 + 5, 0),
                                                    (4099, 0.0, 5, 0), (65537, 0.999, 11, 2 ** 63)])
def test_dropout_mask_bit_exact_and_values(B, count, p, seed, stream_id, dtype):
    rng = np.random.default_rng(2)
    x = rng.standard_normal(count).astype(np.float32) + 3.0      # no zeros: the mask is visible in y
    g = rng.standard_normal(count).astype(np.float32) + 3.0
    if dtype == 1:
        x, g = wl.to_bf16_values(x), wl.to_bf16_values(g)
    y = B.dropout_forward(gpu(x, dtype), p, seed, stream_id)
    dx = B.dropout_backward(gpu(g, dtype), p, seed, stream_id)
    torch.cuda.synchronize()
    p32 = float(np.float32(p))
    keep = oracle.dropout_mask(count, p32, seed, stream_id)
    assert np.array_equal((host(y) != 0).astype(np.uint8), keep)          # integer work: bit-exact
    assert np.array_equal((host(dx) != 0).astype(np.uint8), keep)
    tol = 2e-7 if dtype == 0 else 2.0 ** -8
    for got, src in ((y, x), (dx, g)):
        ref = oracle.dropout_apply(src, p32, seed, stream_id)
        assert np.all(np.abs(host(got) - ref) <= tol * np.abs(ref))
    if p == 0.0:
        assert np.array_equal(host(y), x.astype(np.float64))


def test_dropout_in_place_and_determinism(B):
    x = torch.randn(100001, device="cuda")
    a = B.dropout_forward(x, 0.5, 9, 1)
    b = x.clone()
    B.dropout_forward(b, 0.5, 9, 1, y=b)
    c = B.dropout_forward(x, 0.5, 9, 1)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)
    assert not torch.equal(a, B.dropout_forward(x, 0.5, 10, 1))
    assert B.dropout_forward(torch.empty(0, device="cuda"), 0.5, 1).numel() == 0


def test_whole_caffenet_iteration_small_batch_stage_by_stage(B):
    # conv1..conv5 with pools and normalisation layers, FC6..FC8 with dropout, at batch 4 in bf16: every stage's
    # output and gradient against the oracle applied to what that stage received on the GPU
    from paper_1606_04487_amd.stack import ConvStack
    N, dtype, tol = 4, 1, 2e-2
    layers = wl.caffenet_full(N)
    st = ConvStack(layers, dtype=dtype, ceil_mode=False, skip_first_dgrad=True)
    data = wl.stack_tensors(layers, seed=4, bf16=True, pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    X, dOut = gpu(data["X"], dtype), gpu(data["dY"], dtype)
    out = st.forward(X)
    st.backward(dOut)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (N, 1000, 1, 1)
    h32 = lambda t: t.detach().float().cpu().numpy()

    def close(got, ref, what, limit=tol):
        e = np.max(np.abs(h32(got).astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30)
        assert e <= limit, (what, e)

    size, alpha, beta, k = ConvStack.LRN
    a32 = float(np.float32(alpha))
    g = dOut
    for i in reversed(range(len(layers))):
        L = layers[i]
        s = oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)
        Xi, Wi, Yg = h32(st.X[i]), h32(st.Wc[i]), h32(st.Y[i])
        y_ref = oracle.conv_forward(s, Xi, Wi, data["bias"][i])
        close(st.Y[i], np.maximum(y_ref, 0) if L.relu else y_ref, ("forward", L.name))
        cur = Yg
        if L.pool_after:
            Pref, Aref = oracle.maxpool_forward(Yg, 3, 2, False)
            assert np.array_equal(h32(st.P[i]).astype(np.float64), Pref), ("pool", L.name)
            cur = h32(st.P[i])
        if L.lrn_after:
            close(st.Nrm[i], oracle.lrn_forward(cur, size, a32, beta, k), ("lrn", L.name), 2.0 ** -8)
            lrn_in, cur = cur, h32(st.Nrm[i])
        if L.dropout_after > 0:
            keep = oracle.dropout_mask(cur.size, L.dropout_after, st.dropout_seed, i).reshape(cur.shape)
            # ReLU zeros hide the mask where the input is zero: compare where it is not
            assert np.array_equal((h32(st.Dr[i]) != 0)[cur != 0], keep[cur != 0] == 1), ("dropout mask", L.name)
            close(st.Dr[i], oracle.dropout_apply(cur, L.dropout_after, st.dropout_seed, i), ("dropout", L.name), 2.0 ** -8)
        # backward, in reverse order of the forward stages
        gh = h32(g) if not st.fused_front[i] else None
        if L.dropout_after > 0:
            close(st.gD[i], oracle.dropout_apply(gh, L.dropout_after, st.dropout_seed, i), ("dropout backward", L.name), 2.0 ** -8)
            gh = h32(st.gD[i])
        if L.lrn_after:
            close(st.gN[i], oracle.lrn_backward(lrn_in, gh, size, a32, beta, k), ("lrn backward", L.name), 2.0 ** -7)
            gh = h32(st.gN[i])
        if L.pool_after:
            gh = oracle.maxpool_backward(gh, Aref, L.Ho, L.Wo)
        if not st.fused_front[i]:    # else: checked below, together with the data gradient of the layer behind
            ref_g = oracle.relu_backward(Yg, np.ones_like(Yg)) * gh if L.relu else gh.astype(np.float64)
            close(st.dYc[i], ref_g, ("relu/pool backward", L.name), 2.0 ** -8)
        Gg = h32(st.dYc[i])
        assert np.all(Gg[Yg <= 0] == 0) or not L.relu
        close(st.dW[i], oracle.conv_backward_weights(s, Xi, Gg), ("backward_weights", L.name), 1e-4)
        close(st.db[i], oracle.bias_grad(s, Gg), ("bias gradient", L.name), 1e-4)
        if i > 0 and st.fused_front[i - 1]:
            # this data gradient went out as the front layer's output gradient, its ReLU's mask applied
            Yf = h32(st.Y[i - 1])
            close(st.dYc[i - 1], oracle.conv_backward_data(s, Gg, Wi) * (Yf > 0), ("backward_data + ReLU backward", L.name))
            continue
        if st.dXl[i] is None:
            break
        close(st.dXl[i], oracle.conv_backward_data(s, Gg, Wi), ("backward_data", L.name))
        g = st.dXl[i]
    st.sgd_step(0.01, 0.9)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(w).all()) for w in st.W)
    del st
    torch.cuda.empty_cache()


@pytest.mark.parametrize("g", [2, 4, 8])
def test_implicit_momentum_recursion_through_the_gpu_update(B, g):
    """Sec. IV-C, Theorem 1: g asynchronous groups without explicit momentum behave in expectation like momentum
    SGD with momentum 1 - 1/g and step eta / g.  That recursion, iterated through omni_sgd_momentum_step on a
    quadratic loss (gradients formed on the host from the GPU's current model), must follow the model's own
    reference trajectory."""
    from paper_1606_04487_amd import async_model as am
    A = np.array([[1.0, 0.2], [0.2, 0.5]])
    w_star, w0 = np.array([1.0, -2.0]), np.array([4.0, 3.0])
    eta, steps = 0.4, 80
    # many independent copies of the 2-parameter problem in one tensor, so the launch is not trivially small
    copies = 4096
    W = torch.from_numpy(np.tile(w0, copies).astype(np.float32)).cuda()
    V = torch.zeros_like(W)
    ref = am.implicit_momentum_reference(A, w_star, w0, eta, g, steps)
    for t in range(steps):
        w_host = W.cpu().numpy().astype(np.float64).reshape(copies, 2)
        grad = ((w_host - w_star) @ A.T).astype(np.float32).reshape(-1)
        B.sgd_momentum_step([W], [V], [torch.from_numpy(grad).cuda()], eta / g, 1.0 - 1.0 / g, 0.0)
        got = W.cpu().numpy().reshape(copies, 2)
        assert np.max(np.abs(got - ref[t + 1])) <= 2e-4 * max(1.0, np.max(np.abs(ref[t + 1]))), (g, t)
    # (tests/test_async_model.py checks on the CPU that the asynchronous simulation obeys this recursion step by step)
    assert np.linalg.norm(ref[-1] - w_star) < 0.5 * np.linalg.norm(w0 - w_star)
