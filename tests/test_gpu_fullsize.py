"""GPU parity at the full sizes of the paper's workloads (CaffeNet-shaped layers at batch 256, the
CIFAR-style stack at batch 128), in the launch configuration the bench times.

Whole tensors wherever the direct-loop oracle finishes within a minute on the host: every layer and pass
of the bench configuration (the bf16 stack at batch 256) and of the smaller batches of the sweep, conv1 in
fp32 at batch 256, conv5 alone in both precisions.  The remaining full-size cases compare sampled entries,
which the oracle evaluates one by one (`*_at` routines): random ones plus a fixed set at the places where a
tiling mistake would sit -- both sides of every multiple of the kernels' column tiles (256 / 384 / 512),
the first and last columns, image boundaries, the first and last filters of every 128-row tile, plane
borders.

Two error measures per tensor.  (1) The tensor-normalised one the tolerances are stated in:
max|gpu - ref| / max|ref| <= 1e-4 (fp32) or 2e-2 (bf16).  (2) An elementwise bound that small entries
(borders, where few window taps contribute) cannot hide behind the tensor's maximum:
|gpu - ref| <= tol * S per entry, S = sum of |terms| of that entry (the oracle run on |X|, |W|, |bias|),
and for bf16 outputs additionally the tighter |gpu - ref| <= 2^-8 |ref| + 1e-4 S (one rounding to bf16
plus fp32 accumulation).  The worst ratios are printed (run pytest with -s to see them).

Each stage of a chained stack is compared with the oracle applied to the inputs that stage received on
the GPU.
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


def oshape(L):
    return oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)


# ---------------------------------------------------------------- error measures
def check_errors(what, got, ref, S, tol, rounded_output, s_share=1e-4):
    """Both measures on arrays of equal shape: got (GPU), ref (oracle), S (sum of |terms| per entry).
    s_share: the share of S allowed on top of the output's own rounding in the tighter bf16 bound (1e-4 for
    fp32 accumulation alone; 2^-9 more where partial sums pass through a bf16 matrix, as dD-hat does on the
    explicit data-gradient path before col2im adds its entries)."""
    got = np.asarray(got, dtype=np.float64)
    d = np.abs(got - ref)
    scale = max(float(np.max(np.abs(ref))), 1e-30)
    e_norm = float(np.max(d)) / scale
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(S > 0, d / S, np.where(d > 0, np.inf, 0.0))
    worst = float(np.max(r))
    print(f"{what}: max|d|/max|ref| = {e_norm:.3e} (limit {tol:g}); max |d|/S = {worst:.3e} (limit {tol:g}); "
          f"{got.size} entries")
    assert np.all(np.isfinite(got)), what
    assert e_norm <= tol, (what, "tensor-normalised", e_norm)
    assert worst <= tol, (what, "elementwise |d| <= tol * sum|terms|", worst)
    if rounded_output:
        slack = 2.0 ** -8 * np.abs(ref) + s_share * S - d
        ok = bool(np.all(slack >= 0))
        assert ok, (what, "bf16 rounding + fp32 accumulation bound", float(np.min(slack)))


def edge_values(limit, tiles=(128, 256, 384, 512), ends=16):
    """Indices in [0, limit) where a tiled kernel changes behaviour: both ends and both sides of every tile
    multiple near the start, the middle and the end."""
    pts = set(range(min(ends, limit))) | set(range(max(0, limit - ends), limit))
    for t in tiles:
        n = (limit + t - 1) // t
        for k in {1, 2, n // 2, n - 2, n - 1}:
            for delta in (-1, 0, 1):
                v = k * t + delta
                if 0 <= v < limit:
                    pts.add(v)
    return np.array(sorted(pts), dtype=np.int64)


def boundary_indices(N, F, plane, rows_limit=24):
    """Flat indices into a tensor [N][F][plane]: the edge columns m = n * plane + q of the matrix view
    (tile multiples, first and last columns, image boundaries) crossed with the edge filters."""
    M = N * plane
    cols = set(edge_values(M, tiles=(256, 384, 512), ends=32).tolist())
    for n in {1, 2, N // 2, N - 1}:
        for delta in (-2, -1, 0, 1):
            v = n * plane + delta
            if 0 <= v < M:
                cols.add(v)
    cols = np.array(sorted(cols), dtype=np.int64)
    rows = edge_values(F, tiles=(32, 64, 96, 128), ends=2)[:rows_limit]
    n, q = cols // plane, cols % plane
    idx = (n[None, :] * F + rows[:, None]) * plane + q[None, :]
    return np.unique(idx.reshape(-1))


def sampled(got_tensor, idx):
    flat = got_tensor.detach().reshape(-1)
    return flat[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)


def sample_indices(rng, tensor, fixed):
    rnd = rng.integers(0, tensor.numel(), size=N_SAMPLES)
    return np.unique(np.concatenate([rnd, fixed]))


# ---------------------------------------------------------------- one layer alone
def check_layer(B, L, dtype, seed, x_dist="normal", dgrad=True, whole=False):
    t = wl.layer_tensors(L, seed=seed, x_dist=x_dist, bf16=(dtype == 1))
    s = oshape(L)
    d = B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype)
    X, W, dY, bias = gpu(t["X"], dtype), gpu(t["W"], dtype), gpu(t["dY"], dtype), gpu(t["bias"])
    aX, aW, adY, ab = np.abs(t["X"]), np.abs(t["W"]), np.abs(t["dY"]), np.abs(t["bias"])
    rng = np.random.default_rng(seed + 100)
    nbytes = max(B.conv_workspace_bytes(d, B.PASS_FORWARD), B.conv_workspace_bytes(d, B.PASS_BACKWARD_WEIGHTS))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    tol, rounded = TOL[dtype], dtype == 1
    Y = B.conv_forward(d, X, W, bias, workspace=ws)
    dW, db = B.conv_backward_weights(d.with_flags(B.FLAG_DHAT_CACHED), None, dY, workspace=ws)
    del ws
    dX = B.conv_backward_data(d, dY, W) if dgrad else None
    torch.cuda.synchronize()
    tag = f"{L.name} N={L.N} {'bf16' if dtype else 'fp32'}"
    if whole:
        check_errors(f"{tag} forward (whole)", host32(Y), oracle.conv_forward(s, t["X"], t["W"], t["bias"]),
                     oracle.conv_forward(s, aX, aW, ab), tol, rounded)
        check_errors(f"{tag} backward_weights (whole)", host32(dW), oracle.conv_backward_weights(s, t["X"], t["dY"]),
                     oracle.conv_backward_weights(s, aX, adY), 1e-4, False)
        if dgrad:
            check_errors(f"{tag} backward_data (whole)", host32(dX), oracle.conv_backward_data(s, t["dY"], t["W"]),
                         oracle.conv_backward_data(s, adY, aW), tol, rounded, s_share=1e-4 + 2.0 ** -9)
    else:
        i = sample_indices(rng, Y, boundary_indices(L.N, L.F, L.Ho * L.Wo))
        check_errors(f"{tag} forward (sampled)", sampled(Y, i), oracle.conv_forward_at(s, t["X"], t["W"], t["bias"], i),
                     oracle.conv_forward_at(s, aX, aW, ab, i), tol, rounded)
        i = np.unique(np.concatenate([rng.integers(0, dW.numel(), size=300),
                                      boundary_indices(1, L.F, L.K, rows_limit=8)[::7]]))
        check_errors(f"{tag} backward_weights (sampled)", sampled(dW, i), oracle.conv_backward_weights_at(s, t["X"], t["dY"], i),
                     oracle.conv_backward_weights_at(s, aX, adY, i), 1e-4, False)
        if dgrad:
            i = sample_indices(rng, dX, boundary_indices(L.N, L.C, L.H * L.W))
            check_errors(f"{tag} backward_data (sampled)", sampled(dX, i), oracle.conv_backward_data_at(s, t["dY"], t["W"], i),
                         oracle.conv_backward_data_at(s, adY, aW, i), tol, rounded, s_share=1e-4 + 2.0 ** -9)
    check_errors(f"{tag} bias gradient", host32(db), oracle.bias_grad(s, t["dY"]), oracle.bias_grad(s, adY), 1e-4, False)


def test_caffenet_conv1_fp32_batch256_whole_tensors(B):
    # forward, data gradient and model gradient of the 11x11 stride-4 layer on 256 images, every entry
    check_layer(B, wl.caffenet_stack(256)[0], 0, seed=1, whole=True)


@pytest.mark.parametrize("dtype", [0, 1])
def test_caffenet_conv5_batch256_whole_tensors(B, dtype):
    check_layer(B, wl.caffenet_stack(256)[4], dtype, seed=5, whole=True)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("which", [1, 2, 3])
def test_caffenet_conv2_to_conv4_batch256(B, which, dtype):
    check_layer(B, wl.caffenet_stack(256)[which], dtype, seed=1 + which)


def test_cifar_layers_fp32_batch128(B):
    for i, L in enumerate(wl.cifar_stack(128)):
        check_layer(B, L, 0, seed=10 + i, x_dist="uniform", whole=True)


# ---------------------------------------------------------------- chained stacks
def run_stack(B, layers, dtype, ceil_mode, x_dist, seed, skip_first_dgrad, lr=0.01, mu=0.9):
    """One forward + backward + update of the stack on the GPU; everything read back to the host."""
    from paper_1606_04487_amd.stack import ConvStack
    st = ConvStack(layers, dtype=dtype, ceil_mode=ceil_mode, skip_first_dgrad=skip_first_dgrad)
    data = wl.stack_tensors(layers, seed=seed, x_dist=x_dist, bf16=(dtype == 1), pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    X, dOut = gpu(data["X"], dtype), gpu(data["dY"], dtype)
    st.forward(X)
    st.backward(dOut)
    torch.cuda.synchronize()
    r = {"layers": layers, "dtype": dtype, "ceil_mode": ceil_mode, "bias": data["bias"], "dOut": host32(dOut),
         "X": [host32(x) for x in st.X], "Wc": [host32(w) for w in st.Wc], "Y": [host32(y) for y in st.Y],
         "P": [None if p is None else host32(p) for p in st.P], "dYc": [host32(g) for g in st.dYc],
         "dW": [host32(g) for g in st.dW], "db": [host32(g) for g in st.db],
         "dX": [None if g is None else host32(g) for g in st.dXl], "fused_front": list(st.fused_front),
         "W0": [host32(w) for w in st.W], "b0": [host32(b) for b in st.b]}
    st.sgd_step(lr, mu)
    torch.cuda.synchronize()
    r.update({"W1": [host32(w) for w in st.W], "VW1": [host32(v) for v in st.VW], "b1": [host32(b) for b in st.b],
              "shadow_ok": [dtype != 1 or torch.equal(st.Wc[i], st.W[i].to(torch.bfloat16)) for i in range(len(layers))],
              "lr": lr, "mu": mu})
    del st
    torch.cuda.empty_cache()
    return r


def check_stack_layer(r, i, whole, rng=None):
    """Layer i of a stack run against the oracle applied to what that layer received on the GPU."""
    layers, dtype = r["layers"], r["dtype"]
    L, s, tol, rounded = layers[i], oshape(layers[i]), TOL[dtype], dtype == 1
    Xi, Wi, bi, Yg, Gg = r["X"][i], r["Wc"][i], r["bias"][i], r["Y"][i], r["dYc"][i]
    aX, aW, ab, aG = np.abs(Xi), np.abs(Wi), np.abs(bi), np.abs(Gg)
    # fused_front[i]: this layer's dY came straight out of the data gradient of the layer behind (no dense dX
    # exists); that pair is checked with layer i + 1
    fused_front = r["fused_front"][i]
    g_in = r["dOut"] if i == len(layers) - 1 else (None if fused_front else r["dX"][i + 1])
    tag = f"stack {L.name} N={L.N} {'bf16' if dtype else 'fp32'}"
    rng = rng or np.random.default_rng(1000 + i)
    if whole:
        check_errors(f"{tag} forward+ReLU (whole)", Yg, np.maximum(oracle.conv_forward(s, Xi, Wi, bi), 0),
                     oracle.conv_forward(s, aX, aW, ab), tol, rounded)
    else:
        idx = np.unique(np.concatenate([rng.integers(0, Yg.size, size=N_SAMPLES), boundary_indices(L.N, L.F, L.Ho * L.Wo)]))
        check_errors(f"{tag} forward+ReLU (sampled)", Yg.reshape(-1)[idx], np.maximum(oracle.conv_forward_at(s, Xi, Wi, bi, idx), 0),
                     oracle.conv_forward_at(s, aX, aW, ab, idx), tol, rounded)
    if L.pool_after:
        Pref, Aref = oracle.maxpool_forward(Yg, 3, 2, r["ceil_mode"])
        assert np.array_equal(r["P"][i].astype(np.float64), Pref), ("pool", L.name)
        dYr = oracle.maxpool_backward(g_in, Aref, L.Ho, L.Wo)
        dYa = oracle.maxpool_backward(np.abs(g_in), Aref, L.Ho, L.Wo)
    elif not fused_front:
        dYr = g_in.astype(np.float64)
        dYa = np.abs(dYr)
    # each pixel sums the gradients of the (at most four) windows it won: fp32 on the GPU, rounded once on store;
    # elementwise against the sum of the absolute terms
    mask = oracle.relu_backward(Yg, np.ones_like(Yg))
    tol_g = 1e-6 if dtype == 0 else 2.0 ** -8
    if not fused_front:
        assert np.all(np.abs(Gg - mask * dYr) <= tol_g * mask * dYa), ("relu/pool backward, elementwise", L.name)
    assert np.all(Gg[Yg <= 0] == 0)
    if whole:
        check_errors(f"{tag} backward_weights (whole)", r["dW"][i], oracle.conv_backward_weights(s, Xi, Gg),
                     oracle.conv_backward_weights(s, aX, aG), 1e-4, False)
    else:
        idx = np.unique(np.concatenate([rng.integers(0, r["dW"][i].size, size=200), boundary_indices(1, L.F, L.K, rows_limit=8)[::7]]))
        check_errors(f"{tag} backward_weights (sampled)", r["dW"][i].reshape(-1)[idx], oracle.conv_backward_weights_at(s, Xi, Gg, idx),
                     oracle.conv_backward_weights_at(s, aX, aG, idx), 1e-4, False)
    check_errors(f"{tag} bias gradient", r["db"][i], oracle.bias_grad(s, Gg), oracle.bias_grad(s, aG), 1e-4, False)
    if i > 0 and r["fused_front"][i - 1]:
        # the data gradient went out as the front layer's dY, that layer's ReLU mask applied on the way
        front = r["dYc"][i - 1]
        fmask = (r["Y"][i - 1] > 0).astype(np.float64)
        if whole:
            check_errors(f"{tag} backward_data + ReLU backward (whole)", front, fmask * oracle.conv_backward_data(s, Gg, Wi),
                         fmask * oracle.conv_backward_data(s, aG, aW), tol, rounded)
        else:
            idx = np.unique(np.concatenate([rng.integers(0, front.size, size=N_SAMPLES), boundary_indices(L.N, L.C, L.H * L.W)]))
            m = fmask.reshape(-1)[idx]
            check_errors(f"{tag} backward_data + ReLU backward (sampled)", front.reshape(-1)[idx],
                         m * oracle.conv_backward_data_at(s, Gg, Wi, idx), m * oracle.conv_backward_data_at(s, aG, aW, idx), tol, rounded)
    elif r["dX"][i] is not None:
        if whole:
            check_errors(f"{tag} backward_data (whole)", r["dX"][i], oracle.conv_backward_data(s, Gg, Wi),
                         oracle.conv_backward_data(s, aG, aW), tol, rounded)
        else:
            idx = np.unique(np.concatenate([rng.integers(0, r["dX"][i].size, size=N_SAMPLES), boundary_indices(L.N, L.C, L.H * L.W)]))
            check_errors(f"{tag} backward_data (sampled)", r["dX"][i].reshape(-1)[idx], oracle.conv_backward_data_at(s, Gg, Wi, idx),
                         oracle.conv_backward_data_at(s, aG, aW, idx), tol, rounded)
    # the update of this layer's parameters, whole tensors
    lr, mu = np.float32(r["lr"]), np.float32(r["mu"])
    W1, V1 = oracle.sgd_momentum(r["W0"][i], np.zeros_like(r["W0"][i]), r["dW"][i], lr, mu, 0.0)
    b1, _ = oracle.sgd_momentum(r["b0"][i], np.zeros_like(r["b0"][i]), r["db"][i], lr, mu, 0.0)
    assert np.max(np.abs(r["W1"][i] - W1)) <= 1e-6 * np.max(np.abs(W1))
    assert np.max(np.abs(r["VW1"][i] - V1)) <= 1e-6 * max(np.max(np.abs(V1)), 1e-30)
    assert np.max(np.abs(r["b1"][i] - b1)) <= 1e-6 * np.max(np.abs(b1))
    assert r["shadow_ok"][i]


def check_stack(B, layers, dtype, ceil_mode, x_dist, seed, skip_first_dgrad, whole):
    r = run_stack(B, layers, dtype, ceil_mode, x_dist, seed, skip_first_dgrad)
    rng = np.random.default_rng(seed + 7)
    for i in reversed(range(len(layers))):
        check_stack_layer(r, i, whole, rng)


def test_cifar_stack_fp32_batch128(B):
    check_stack(B, wl.cifar_stack(128), 0, True, "uniform", seed=1, skip_first_dgrad=False, whole=True)


@pytest.mark.parametrize("dtype", [0, 1])
def test_caffenet_conv2_to_conv5_chained_batch256(B, dtype):
    layers = wl.caffenet_stack(256)[1:]
    check_stack(B, layers, dtype, False, "normal", seed=2, skip_first_dgrad=False, whole=False)


@pytest.mark.parametrize("N", [1, 16, 64])
def test_caffenet_full_stack_bf16_small_batches_whole_tensors(B, N):
    # the smaller batches of the sweep, every entry of every tensor
    check_stack(B, wl.caffenet_stack(N), 1, False, "normal", seed=3, skip_first_dgrad=True, whole=True)


@pytest.fixture(scope="module")
def bench_run(B):
    # the configuration the bench times: conv1..conv5 at batch 256, bf16, conv1's data gradient skipped
    return run_stack(B, wl.caffenet_stack(256), 1, False, "normal", seed=3, skip_first_dgrad=True)


@pytest.mark.parametrize("i", [4, 3, 2, 1, 0])
def test_bench_configuration_batch256_whole_tensors(bench_run, i):
    # one test per layer so that none runs the oracle for more than about a minute
    check_stack_layer(bench_run, i, whole=True)


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
