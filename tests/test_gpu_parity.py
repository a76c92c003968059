"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element.

Tolerances (tensor-normalised: max|gpu - ref| / max|ref|): 1e-4 for fp32 storage, 2e-2 for bf16
storage.  Lowering, pooling values/argmax and ReLU are pure copies/selections and must be
bit-exact; col2im is checked bit-exactly on small-integer data (every partial sum is exact).
bf16 cases feed both sides the same bf16-representable values; the oracle accumulates in fp64.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


def gpu(a, dtype=0):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == 1 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    scale = np.max(np.abs(ref))
    return np.max(np.abs(got - ref)) / (scale if scale > 0 else 1.0)


def prep(a, dtype):
    return wl.to_bf16_values(a) if dtype == 1 else np.ascontiguousarray(a, dtype=np.float32)


# (N, C, H, W, F, kh, kw, sh, sw, ph, pw): sizes that span several 128-wide tiles with ragged tails,
# every stride/pad combination of the paper's layers, and degenerate extents.
SHAPES = [
    (8, 3, 32, 32, 32, 5, 5, 1, 1, 2, 2),       # the small single-layer configuration
    (3, 5, 13, 13, 7, 3, 3, 1, 1, 1, 1),        # M = 507 (not a multiple of 8), K = 45, F = 7
    (2, 3, 35, 35, 96, 11, 11, 4, 4, 0, 0),     # conv1-like: stride 4, K = 363
    (2, 20, 27, 27, 130, 5, 5, 1, 1, 2, 2),     # F = 130: two row tiles, second nearly empty
    (1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0),          # one element
    (2, 4, 9, 7, 5, 3, 2, 2, 1, 1, 0),          # non-square everything
    (5, 40, 13, 13, 200, 3, 3, 1, 1, 1, 1),     # K = 360, M = 845
    (1, 2, 6, 6, 3, 3, 3, 1, 1, 3, 3),          # pad >= kernel
    (4, 16, 8, 8, 64, 5, 5, 1, 1, 2, 2),        # CIFAR conv3-like
]


def make(cfg, dtype, seed=0):
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
    ho, wo = oracle.out_dims(s)
    rng = np.random.default_rng(seed)
    X = prep(rng.standard_normal((N, C, H, W)), dtype)
    Wt = prep(0.05 * rng.standard_normal((F, C, kh, kw)), dtype)
    b = (0.05 * rng.standard_normal(F)).astype(np.float32)
    dY = prep(rng.standard_normal((N, F, ho, wo)), dtype)
    return s, X, Wt, b, dY


def desc_of(B, cfg, dtype, flags=0):
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    return B.conv_desc(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw), dtype, flags)


# ------------------------------------------------------------------------------------ lowering

@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", SHAPES)
def test_lower_bit_exact(B, cfg, dtype):
    s, X, *_ = make(cfg, dtype, 1)
    d = desc_of(B, cfg, dtype)
    ref = oracle.lower(s, X)
    M = ref.shape[1]
    got = B.lower(d, gpu(X, dtype))                       # canonical leading dimension M
    assert np.array_equal(host(got).astype(np.float32).view(np.uint32), ref.view(np.uint32))
    ld = B.conv_dhat_ld(d) + 8                            # padded: extra columns must be zero
    got = B.lower(d, gpu(X, dtype), ld=ld)
    g = host(got).astype(np.float32)
    assert np.array_equal(g[:, :M].view(np.uint32), ref.view(np.uint32))
    assert np.all(g[:, M:].view(np.uint32) == 0)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", SHAPES)
def test_col2im(B, cfg, dtype):
    s, *_ = make(cfg, dtype, 2)
    d = desc_of(B, cfg, dtype)
    ho, wo = oracle.out_dims(s)
    K, M = s.C * s.kh * s.kw, s.N * ho * wo
    rng = np.random.default_rng(3)
    Zi = rng.integers(-3, 4, size=(K, M)).astype(np.float32)      # integer data: sums are exact
    got = B.col2im(d, gpu(Zi, dtype))
    assert np.array_equal(host(got), oracle.col2im(s, Zi))
    Z = prep(rng.standard_normal((K, M)), dtype)
    ld = M + 5
    Zp = np.concatenate([Z, np.full((K, 5), 7.0, np.float32)], axis=1)   # columns >= M must be ignored
    got = B.col2im(d, gpu(Zp, dtype), ld=ld)
    assert rel_err(host(got), oracle.col2im(s, Z)) <= TOL[dtype]


# Strided layers whose per-image segments exceed what the LDS-staged kernel holds (or whose leading dimension is
# not a multiple of the vector width) take the form with S pixels per thread: strides 2 and 4, windows with one to
# three taps per pixel and direction, widths that are not multiples of the stride, padding.
STRIDED = [
    (2, 2, 65, 65, 1, 7, 7, 2, 2, 3, 3),
    (1, 2, 115, 113, 1, 11, 11, 4, 4, 0, 0),
    (1, 2, 137, 135, 1, 3, 3, 2, 2, 1, 1),
    (2, 3, 40, 38, 1, 5, 12, 4, 4, 2, 5),
    (3, 2, 21, 23, 1, 4, 4, 4, 4, 0, 0),
    (2, 2, 19, 18, 1, 2, 6, 2, 2, 0, 2),
]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", STRIDED)
def test_col2im_strided(B, cfg, dtype):
    s, *_ = make(cfg, dtype, 4)
    d = desc_of(B, cfg, dtype)
    ho, wo = oracle.out_dims(s)
    K, M = s.C * s.kh * s.kw, s.N * ho * wo
    rng = np.random.default_rng(5)
    Zi = rng.integers(-3, 4, size=(K, M)).astype(np.float32)      # integer data: sums are exact
    ref = oracle.col2im(s, Zi)
    for pad in (0, 3):
        Zp = np.concatenate([Zi, np.full((K, pad), 7.0, np.float32)], axis=1) if pad else Zi
        got = B.col2im(d, gpu(Zp, dtype), ld=M + pad)
        assert np.array_equal(host(got), ref), (cfg, pad)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", STRIDED + [(1, 2, 150, 9, 1, 3, 3, 1, 1, 1, 1), (1, 1, 97, 200, 1, 5, 5, 1, 1, 2, 2)])
def test_lower_large_planes(B, cfg, dtype):
    """Planes too large for whole images per workgroup: bands of output rows, narrow bands with the threads split
    into row groups."""
    s, X, *_ = make(cfg, dtype, 6)
    d = desc_of(B, cfg, dtype)
    ref = oracle.lower(s, X)
    M = ref.shape[1]
    for pad in (0, 16, 3):
        got = host(B.lower(d, gpu(X, dtype), ld=M + pad)).astype(np.float32)
        assert np.array_equal(got[:, :M].view(np.uint32), ref.view(np.uint32)), (cfg, pad)
        assert np.all(got[:, M:].view(np.uint32) == 0)


# ------------------------------------------------------------------------------------ the three passes

@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", SHAPES)
def test_conv_forward(B, cfg, dtype):
    s, X, Wt, b, _ = make(cfg, dtype, 4)
    d = desc_of(B, cfg, dtype)
    Xg, Wg, bg = gpu(X, dtype), gpu(Wt, dtype), gpu(b)
    ref = oracle.conv_forward(s, X, Wt, b)
    assert rel_err(host(B.conv_forward(d, Xg, Wg, bg)), ref) <= TOL[dtype]
    ref_nb = oracle.conv_forward(s, X, Wt, None)
    assert rel_err(host(B.conv_forward(d, Xg, Wg, None)), ref_nb) <= TOL[dtype]
    dr = desc_of(B, cfg, dtype, B.FLAG_RELU)
    got = host(B.conv_forward(dr, Xg, Wg, bg))
    assert rel_err(got, np.maximum(ref, 0)) <= TOL[dtype]
    assert got.min() >= 0


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", SHAPES)
def test_conv_backward_data(B, cfg, dtype):
    s, X, Wt, b, dY = make(cfg, dtype, 5)
    d = desc_of(B, cfg, dtype)
    got = B.conv_backward_data(d, gpu(dY, dtype), gpu(Wt, dtype))
    assert rel_err(host(got), oracle.conv_backward_data(s, dY, Wt)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", SHAPES)
def test_conv_backward_weights(B, cfg, dtype):
    s, X, Wt, b, dY = make(cfg, dtype, 6)
    d = desc_of(B, cfg, dtype)
    dW, db = B.conv_backward_weights(d, gpu(X, dtype), gpu(dY, dtype))
    assert dW.dtype == torch.float32 and db.dtype == torch.float32
    assert rel_err(host(dW), oracle.conv_backward_weights(s, X, dY)) <= 1e-4     # fp32 out in both modes
    assert rel_err(host(db), oracle.bias_grad(s, dY)) <= 1e-4
    dW2, none = B.conv_backward_weights(d, gpu(X, dtype), gpu(dY, dtype), want_dbias=False)
    assert none is None and torch.equal(dW, dW2)


@pytest.mark.parametrize("dtype", [0, 1])
def test_cached_dhat_and_determinism(B, dtype):
    cfg = SHAPES[3]
    s, X, Wt, b, dY = make(cfg, dtype, 7)
    d = desc_of(B, cfg, dtype)
    Xg, Wg, bg, Gg = gpu(X, dtype), gpu(Wt, dtype), gpu(b), gpu(dY, dtype)
    nbytes = max(B.conv_workspace_bytes(d, B.PASS_FORWARD), B.conv_workspace_bytes(d, B.PASS_BACKWARD_WEIGHTS))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Y1 = B.conv_forward(d, Xg, Wg, bg, workspace=ws)
    dW1, db1 = B.conv_backward_weights(d.with_flags(B.FLAG_DHAT_CACHED), None, Gg, workspace=ws)
    dW2, db2 = B.conv_backward_weights(d, Xg, Gg)
    assert torch.equal(dW1, dW2) and torch.equal(db1, db2)
    Y2 = B.conv_forward(d, Xg, Wg, bg)
    dX1, dX2 = B.conv_backward_data(d, Gg, Wg), B.conv_backward_data(d, Gg, Wg)
    assert torch.equal(Y1, Y2) and torch.equal(dX1, dX2)       # run-to-run bit-identical


def test_adjoint_identities_on_gpu(B):
    # <conv(X,W), G> = <X, dgrad(G,W)> = <W, wgrad(X,G)> evaluated from GPU results (fp32).
    cfg = (4, 24, 27, 27, 96, 5, 5, 1, 1, 2, 2)
    s, X, Wt, b, dY = make(cfg, 0, 8)
    d = desc_of(B, cfg, 0)
    Xg, Wg, Gg = gpu(X), gpu(Wt), gpu(dY)
    Y = host(B.conv_forward(d, Xg, Wg, None))
    dX = host(B.conv_backward_data(d, Gg, Wg))
    dW = host(B.conv_backward_weights(d, Xg, Gg)[0])
    a = np.sum(Y * dY)
    assert abs(a - np.sum(X * dX)) <= 1e-4 * abs(a) + 1e-2
    assert abs(a - np.sum(Wt * dW)) <= 1e-4 * abs(a) + 1e-2


# ------------------------------------------------------------------------------------ update and glue

def test_sgd_momentum_step(B):
    rng = np.random.default_rng(9)
    sizes = [1, 3, 4, 5, 1023, 4096, 4097, 34848, 100003] + [17] * 30      # > one table of tensors
    W0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    V0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    G = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    Wg, Vg, Gg = [gpu(a) for a in W0], [gpu(a) for a in V0], [gpu(a) for a in G]
    Sg = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") if i % 2 == 0 else None for i, n in enumerate(sizes)]
    B.sgd_momentum_step(Wg, Vg, Gg, 0.01, 0.9, 5e-4, Sg)
    for i in range(len(sizes)):
        W1, V1 = oracle.sgd_momentum(W0[i], V0[i], G[i], np.float32(0.01), np.float32(0.9), np.float32(5e-4))
        assert rel_err(host(Wg[i]), W1) <= 1e-6 and rel_err(host(Vg[i]), V1) <= 1e-6
        if Sg[i] is not None:
            assert torch.equal(Sg[i], Wg[i].to(torch.bfloat16))
    # Eq. (update2)/(update1) from V = 0 with lr 0.01, mu 0.9: V = -0.01 G exactly representable check
    W, V, Gc = gpu(np.ones(8)), gpu(np.zeros(8)), gpu(np.full(8, 2.0))
    B.sgd_momentum_step([W], [V], [Gc], 0.5, 0.5)
    assert np.array_equal(host(V), np.full(8, -1.0)) and np.array_equal(host(W), np.zeros(8))
    B.sgd_momentum_step([], [], [], 0.1, 0.9)               # empty list: no-op
    B.sgd_momentum_step([torch.zeros(0, device="cuda")], [torch.zeros(0, device="cuda")],
                        [torch.zeros(0, device="cuda")], 0.1, 0.9)


@pytest.mark.parametrize("dtype", [0, 1])
def test_relu(B, dtype):
    for n in (1, 7, 8, 1000, 4099):
        x = prep(np.random.default_rng(n).standard_normal(n), dtype)
        x[::5] = 0.0
        dy = prep(np.random.default_rng(n + 1).standard_normal(n), dtype)
        y = B.relu_forward(gpu(x, dtype))
        assert np.array_equal(host(y), oracle.relu_forward(x))
        dx = B.relu_backward(y, gpu(dy, dtype))
        assert np.array_equal(host(dx), oracle.relu_backward(x, dy))
    B.relu_forward(torch.zeros(0, device="cuda"))


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("H,W,ceil_mode", [(32, 32, True), (32, 32, False), (16, 16, True), (8, 8, True),
                                            (55, 55, True), (13, 13, False), (7, 9, True), (3, 3, True),
                                            (27, 27, True), (6, 20, True), (5, 14, False), (9, 11, True),
                                            (4, 10, True), (5, 17, False), (12, 29, True)])
def test_maxpool(B, dtype, H, W, ceil_mode):
    rng = np.random.default_rng(H * 100 + W)
    x = prep(rng.standard_normal((3, 5, H, W)), dtype)
    if dtype == 1:
        x = prep(np.round(x * 2) / 2, dtype)        # many exact ties: the first maximum must win
    y_ref, am_ref = oracle.maxpool_forward(x, 3, 2, ceil_mode)
    y, am = B.maxpool_forward(gpu(x, dtype), 3, 2, ceil_mode)
    assert np.array_equal(host(y), y_ref)
    ho, wo = y_ref.shape[-2:]
    code = am.cpu().numpy().astype(np.int64)
    oy, ox = np.meshgrid(np.arange(ho), np.arange(wo), indexing="ij")
    flat = (oy * 2 + code // 3) * W + (ox * 2 + code % 3)
    assert np.array_equal(flat, am_ref)
    dy = prep(rng.standard_normal(y_ref.shape), dtype)
    dx = B.maxpool_backward(gpu(dy, dtype), am, H, W, 3, 2, ceil_mode)
    ref = oracle.maxpool_backward(dy, am_ref, H, W)
    if dtype == 0:
        assert rel_err(host(dx), ref) <= 1e-6
    else:
        assert rel_err(host(dx), ref) <= TOL[1]
    # fused with the gradient of a ReLU in front of the pool (mask taken from the pooled values): exactly
    # the unfused result where x > 0, else 0
    fused = B.maxpool_relu_backward(gpu(dy, dtype), am, gpu(y_ref, dtype), H, W, 3, 2, ceil_mode)
    expect = torch.where(gpu(x, dtype) > 0, dx, torch.zeros_like(dx))
    assert torch.equal(fused, expect)
    assert np.array_equal(host(fused) != 0, (oracle.relu_backward(x, np.ones_like(x)) * ref) != 0) or dtype == 1


@pytest.mark.parametrize("H,W,ceil_mode", [(55, 55, True), (27, 27, True), (13, 13, False), (7, 9, True), (3, 3, True),
                                            (6, 20, True), (5, 14, False), (12, 29, True), (4, 4, True)])
def test_maxpool_forward_kernels_agree(B, H, W, ceil_mode):
    """bf16 3 x 3 / stride 2 forward pool: the kernel that reads the planes directly (the default) and the one that
    stages them in LDS give the same values and winners, also where -0 and +0 tie and at the tensor's last rows
    (where the direct kernel's loads are moved back to stay inside the tensor); both equal the oracle."""
    rng = np.random.default_rng(H * 37 + W)
    x = prep(np.round(rng.standard_normal((2, 3, H, W)) * 2) / 2, 1)
    xg = gpu(x, 1)
    try:
        B.tuning_set(B.TUNE_POOL_LDS, 1)
        y_lds, am_lds = B.maxpool_forward(xg, 3, 2, ceil_mode)
        B.tuning_set(B.TUNE_POOL_LDS, 0)
        y_dir, am_dir = B.maxpool_forward(xg, 3, 2, ceil_mode)
    finally:
        B.tuning_set(B.TUNE_POOL_LDS, 0)
    assert torch.equal(y_lds.view(torch.int16), y_dir.view(torch.int16)) and torch.equal(am_lds, am_dir)
    y_ref, am_ref = oracle.maxpool_forward(x, 3, 2, ceil_mode)
    assert np.array_equal(host(y_dir), y_ref)
    no_winners = B.maxpool_forward(xg, 3, 2, ceil_mode, argmax=None)[0]
    assert torch.equal(no_winners, y_dir)


# ------------------------------------------------------------------------------------ chained stack

@pytest.mark.parametrize("dtype", [0, 1])
def test_cifar_stack_layer_by_layer(B, dtype):
    """CIFAR-style stack, forward + backward + one momentum step; every stage is compared with the
    oracle applied to the inputs that stage actually received on the GPU."""
    from paper_1606_04487_amd.stack import ConvStack
    N = 16
    layers = wl.cifar_stack(N)
    st = ConvStack(layers, dtype=dtype, skip_first_dgrad=False)
    data = wl.stack_tensors(layers, seed=1, x_dist="uniform", bf16=(dtype == 1), pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    X, dOut = gpu(data["X"], dtype), gpu(data["dY"], dtype)
    out = st.forward(X)
    assert tuple(out.shape) == (N, 64, 4, 4)
    dX = st.backward(dOut)
    tol = TOL[dtype]
    g_in = dOut
    for i in reversed(range(3)):
        L = layers[i]
        s = oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)
        Xi, Wi = host(st.X[i]), host(st.Wc[i])
        Yref = np.maximum(oracle.conv_forward(s, Xi, Wi, data["bias"][i]), 0)
        assert rel_err(host(st.Y[i]), Yref) <= tol
        Yg = host(st.Y[i])
        Pref, Aref = oracle.maxpool_forward(Yg, 3, 2, True)
        assert np.array_equal(host(st.P[i]), Pref)
        dYr = oracle.maxpool_backward(host(g_in), Aref, L.Ho, L.Wo)
        dYc = oracle.relu_backward(Yg, dYr)
        assert rel_err(host(st.dYc[i]), dYc) <= tol
        G = host(st.dYc[i])
        assert rel_err(host(st.dW[i]), oracle.conv_backward_weights(s, Xi, G)) <= 1e-4
        assert rel_err(host(st.db[i]), oracle.bias_grad(s, G)) <= 1e-4
        assert rel_err(host(st.dXl[i]), oracle.conv_backward_data(s, G, Wi)) <= tol
        g_in = st.dXl[i]
    # one momentum step from V = 0 (lr 0.01, mu 0.9): V = -0.01 G, W = W0 + V
    W0 = [host(w) for w in st.W]
    dW = [host(g) for g in st.dW]
    st.sgd_step(0.01, 0.9)
    for i in range(3):
        W1, V1 = oracle.sgd_momentum(W0[i], np.zeros_like(W0[i]), dW[i], np.float32(0.01), np.float32(0.9), 0.0)
        assert rel_err(host(st.W[i]), W1) <= 1e-6 and rel_err(host(st.VW[i]), V1) <= 1e-6
        if dtype == 1:
            assert torch.equal(st.Wc[i], st.W[i].to(torch.bfloat16))


# ------------------------------------------------------------------------------------ error paths on device

def test_workspace_too_small_and_misaligned(B):
    cfg = SHAPES[0]
    s, X, Wt, b, dY = make(cfg, 0, 11)
    d = desc_of(B, cfg, 0)
    Xg, Wg = gpu(X), gpu(Wt)
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.OmniError) as e:
        B.conv_forward(d, Xg, Wg, None, workspace=small)
    assert e.value.status == -3
    ws = torch.empty(B.conv_workspace_bytes(d, B.PASS_FORWARD) + 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.OmniError) as e:
        B.conv_forward(d, Xg, Wg, None, workspace=ws[4:])
    assert e.value.status == -4


# ------------------------------------------------------------------------------------ partial batching

@pytest.mark.parametrize("dtype", [0, 1])
def test_partial_batching_gives_identical_results(B, dtype):
    """Sec. III-B: lowering and multiplying b_p images at a time changes memory and speed, not the result."""
    cfg = (12, 8, 13, 13, 24, 3, 3, 1, 1, 1, 1)
    s, X, Wt, b, _ = make(cfg, dtype, 21)
    d = desc_of(B, cfg, dtype, B.FLAG_RELU)
    Xg, Wg, bg = gpu(X, dtype), gpu(Wt, dtype), gpu(b)
    whole = B.conv_forward(d, Xg, Wg, bg)
    assert rel_err(host(whole), np.maximum(oracle.conv_forward(s, X, Wt, b), 0)) <= TOL[dtype]
    for bp in (1, 2, 5, 6, 12):                      # 5 does not divide 12: a smaller last group
        part = B.conv_forward_partial(d, bp, Xg, Wg, bg)
        assert torch.equal(part, whole), bp


# ------------------------------------------------------------------------------------ fully connected layers

@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", [(16, 64, 6, 6, 136, 6, 6, 1, 1, 0, 0),     # FC6-like: the window covers the whole image
                                 (40, 200, 1, 1, 72, 1, 1, 1, 1, 0, 0)])   # FC7/8-like: 1 x 1 images
def test_fully_connected_as_convolution(B, cfg, dtype):
    """Sec. II-C: a fully connected layer is a dense matrix product; it is the convolution whose window is
    the whole image (App. C's m = n - k + 1 = 1), so the same three entry points serve the FC phase."""
    s, X, Wt, b, dY = make(cfg, dtype, 31)
    d = desc_of(B, cfg, dtype)
    Xg, Wg, bg, dYg = gpu(X, dtype), gpu(Wt, dtype), gpu(b), gpu(dY, dtype)
    N, C, H, W, F = cfg[:5]
    Y = B.conv_forward(d, Xg, Wg, bg)
    ref = X.reshape(N, -1).astype(np.float64) @ Wt.reshape(F, -1).astype(np.float64).T + b      # the plain definition
    assert rel_err(host(Y).reshape(N, F), ref) <= TOL[dtype]
    assert rel_err(host(Y), oracle.conv_forward(s, X, Wt, b)) <= TOL[dtype]
    dX = B.conv_backward_data(d, dYg, Wg)
    assert rel_err(host(dX).reshape(N, -1), dY.reshape(N, F).astype(np.float64) @ Wt.reshape(F, -1)) <= TOL[dtype]
    dW, db = B.conv_backward_weights(d, Xg, dYg)
    assert rel_err(host(dW).reshape(F, -1), dY.reshape(N, F).astype(np.float64).T @ X.reshape(N, -1)) <= 1e-4
    assert rel_err(host(db), dY.reshape(N, F).sum(0)) <= 1e-4


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("cfg", [(16, 64, 6, 6, 136, 6, 6, 1, 1, 0, 0),      # FC6-like: 2304-long reduction, 16 columns
                                 (24, 1200, 1, 1, 72, 1, 1, 1, 1, 0, 0),    # FC7/8-like
                                 (1, 48, 13, 13, 64, 5, 5, 1, 1, 2, 2),     # one image per product (b_p = 1)
                                 (4, 16, 4, 4, 1024, 3, 3, 1, 1, 1, 1),     # many filters: the data gradient's reduction splits
                                 (8, 32, 2, 2, 2048, 2, 2, 1, 1, 0, 0)])    # whole-image window: the dense data gradient, split
def test_split_reduction(B, cfg, dtype):
    """OMNI_FLAG_SPLIT_K: products with few columns split their reduction over the chip.  Same bars as the
    unsplit products against the oracle, agreement with them to rounding, deterministic, and the extra
    workspace is accounted for."""
    s, X, Wt, b, dY = make(cfg, dtype, 41)
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    plain = desc_of(B, cfg, dtype)
    split = B.conv_desc(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw), dtype, B.FLAG_SPLIT_K | B.FLAG_RELU)
    assert B.conv_workspace_bytes(split, B.PASS_FORWARD) >= B.conv_workspace_bytes(plain, B.PASS_FORWARD)
    Xg, Wg, bg, dYg = gpu(X, dtype), gpu(Wt, dtype), gpu(b), gpu(dY, dtype)
    Y = B.conv_forward(split, Xg, Wg, bg)
    ref = np.maximum(oracle.conv_forward(s, X, Wt, b), 0)
    assert rel_err(host(Y), ref) <= TOL[dtype]
    Y0 = B.conv_forward(plain.with_flags(B.FLAG_RELU), Xg, Wg, bg)
    assert rel_err(host(Y), host(Y0)) <= (1e-5 if dtype == 0 else 1e-2)
    assert torch.equal(Y, B.conv_forward(split, Xg, Wg, bg))
    dX = B.conv_backward_data(split, dYg, Wg)
    assert rel_err(host(dX), oracle.conv_backward_data(s, dY, Wt)) <= TOL[dtype]
    assert rel_err(host(dX), host(B.conv_backward_data(plain, dYg, Wg))) <= (1e-5 if dtype == 0 else 1e-2)
    assert torch.equal(dX, B.conv_backward_data(split, dYg, Wg))
    # the model gradient ignores the flag
    dW, _ = B.conv_backward_weights(split, Xg, dYg)
    dW0, _ = B.conv_backward_weights(plain, Xg, dYg)
    assert torch.equal(dW, dW0)
