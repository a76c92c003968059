"""Pins for the CPU oracle: closed forms, invariants, library routines and brute force.

Nothing here compares the oracle with itself by retyping its formula: every expected value
comes from a closed form, an algebraic identity, an independently written route (pure-Python
index loops + numpy matmul), or a library routine (torch's CPU float64 convolution, unfold,
fold, max_pool2d and autograd).  Passages: Sec. II-B (BW, update equations), Sec. III-A
Eq. (conv_full), App. C (lowering, m = n-k+1, replication m^2 k^2 / n^2), Sec. II-C and
App. B (1.6 TFLOP rule).
"""
import itertools
import os
import re

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

import oracle
from oracle import lowering_route as lr
from paper_1606_04487_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")

# (N, C, H, W, F, kh, kw, sh, sw, ph, pw): tiny, deliberately lopsided shapes
TINY = [
    (1, 1, 5, 5, 1, 3, 3, 1, 1, 0, 0),
    (2, 3, 7, 6, 4, 3, 2, 1, 1, 1, 0),
    (2, 2, 7, 7, 3, 5, 5, 1, 1, 2, 2),
    (1, 3, 9, 8, 2, 3, 3, 2, 2, 1, 1),
    (2, 2, 11, 11, 3, 3, 3, 4, 4, 0, 0),
    (1, 2, 8, 10, 3, 2, 3, 2, 1, 0, 2),
    (2, 1, 6, 6, 2, 1, 1, 1, 1, 0, 0),
    (1, 2, 5, 7, 2, 3, 3, 1, 2, 2, 1),
    (1, 3, 12, 12, 2, 5, 5, 4, 4, 0, 0),
    (2, 2, 4, 4, 2, 3, 3, 1, 1, 3, 3),      # pad >= kernel: rows of pure padding
]


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _mk(cfg, seed=0):
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
    ho, wo = oracle.out_dims(s)
    X = _rand((N, C, H, W), seed)
    Wt = _rand((F, C, kh, kw), seed + 1)
    b = _rand((F,), seed + 2)
    dY = _rand((N, F, ho, wo), seed + 3)
    return s, X, Wt, b, dY


def _facts():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


# ----------------------------------------------------------------------------- forward

def test_centred_delta_kernel_is_identity():
    # Eq. (conv_full) with K = delta at the window centre, stride 1, pad k/2: R == D exactly.
    for k in (1, 3, 5):
        C = 3
        s = oracle.shape(2, C, 6, 7, C, k, k, 1, k // 2)
        X = _rand((2, C, 6, 7), 5)
        Wt = np.zeros((C, C, k, k), np.float32)
        for c in range(C):
            Wt[c, c, k // 2, k // 2] = 1.0
        Y = oracle.conv_forward(s, X, Wt)
        assert np.array_equal(Y, X.astype(np.float64))


@pytest.mark.parametrize("ky,kx", [(0, 0), (0, 2), (2, 0), (1, 2), (2, 2)])
def test_shifted_delta_pins_no_flip_and_pad_direction(ky, kx):
    # A delta at (ky,kx) must give Y[oy,ox] = X[oy-p+ky, ox-p+kx] with zero fill: this fails for
    # a flipped kernel, a swapped x/y, or padding applied on the wrong side.
    k, p, H, W = 3, 1, 5, 6
    s = oracle.shape(1, 1, H, W, 1, k, k, 1, p)
    X = _rand((1, 1, H, W), 9)
    Wt = np.zeros((1, 1, k, k), np.float32)
    Wt[0, 0, ky, kx] = 1.0
    Y = oracle.conv_forward(s, X, Wt)[0, 0]
    Xp = np.zeros((H + 2 * p, W + 2 * p))
    Xp[p:p + H, p:p + W] = X[0, 0]
    expect = Xp[ky:ky + H, kx:kx + W]
    assert np.array_equal(Y, expect)


@pytest.mark.parametrize("cfg", TINY)
def test_all_ones_counts_in_range_taps(cfg):
    # X == 1, W == 1: each output is C * (#taps inside the image), a product of per-axis counts.
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
    ho, wo = oracle.out_dims(s)
    Y = oracle.conv_forward(s, np.ones((N, C, H, W), np.float32), np.ones((F, C, kh, kw), np.float32))
    cy = np.array([sum(0 <= oy * sh - ph + t < H for t in range(kh)) for oy in range(ho)])
    cx = np.array([sum(0 <= ox * sw - pw + t < W for t in range(kw)) for ox in range(wo)])
    expect = C * np.outer(cy, cx)
    assert np.array_equal(Y, np.broadcast_to(expect, Y.shape))
    if ph == 0 and pw == 0:
        assert np.all(Y == C * kh * kw)


def test_valid_extent_is_n_minus_k_plus_1():
    assert _facts()["valid_output_extent"] == "n - k + 1"   # App. C
    for n, k in itertools.product((5, 13, 27, 227), (1, 3, 5, 11)):
        if n < k:
            continue
        assert oracle.out_dims(oracle.shape(1, 1, n, n, 1, k)) == (n - k + 1, n - k + 1)
    # the CaffeNet shapes this build runs
    assert [(L.Ho, L.Wo) for L in wl.caffenet_stack()] == [(55, 55), (27, 27), (13, 13), (13, 13), (13, 13)]
    with pytest.raises(ValueError):
        oracle.out_dims(oracle.shape(1, 1, 3, 3, 1, 5))      # window larger than the image


@pytest.mark.parametrize("cfg", TINY)
def test_linearity(cfg):
    s, X, Wt, b, _ = _mk(cfg, 20)
    X2, W2 = _rand(X.shape, 31), _rand(Wt.shape, 32)
    # exact float arithmetic on small integers keeps the identities free of rounding
    Xi, X2i = np.round(X * 4), np.round(X2 * 4)
    Wi, W2i = np.round(Wt * 4), np.round(W2 * 4)
    f = oracle.conv_forward
    assert np.array_equal(f(s, Xi + X2i, Wi), f(s, Xi, Wi) + f(s, X2i, Wi))
    assert np.array_equal(f(s, Xi, Wi + W2i), f(s, Xi, Wi) + f(s, Xi, W2i))
    assert np.array_equal(f(s, 3 * Xi, Wi), 3 * f(s, Xi, Wi))
    bi = np.round(b * 4)
    assert np.array_equal(f(s, Xi, Wi, bi), f(s, Xi, Wi) + bi[None, :, None, None])


@pytest.mark.parametrize("cfg", TINY)
def test_direct_loops_match_lowering_route(cfg):
    # App. C: lowering + GEMM + lifting regroups the same sum.
    s, X, Wt, b, dY = _mk(cfg, 40)
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    np.testing.assert_allclose(oracle.conv_forward(s, X, Wt, b),
                               lr.conv_forward(X, Wt, b, sh, sw, ph, pw), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_backward_data(s, dY, Wt),
                               lr.conv_backward_data(dY, Wt, H, W, sh, sw, ph, pw), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_backward_weights(s, X, dY),
                               lr.conv_backward_weights(X, dY, kh, kw, sh, sw, ph, pw), rtol=0, atol=1e-12)


@pytest.mark.parametrize("cfg", TINY + [(3, 4, 13, 13, 6, 3, 3, 1, 1, 1, 1), (2, 3, 35, 35, 5, 11, 11, 4, 4, 0, 0)])
def test_against_torch_float64_convolution_and_autograd(cfg):
    # Library routine: torch's CPU conv2d in float64 and its autograd gradients.
    s, X, Wt, b, dY = _mk(cfg, 60)
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    Xt = torch.from_numpy(X).double().requires_grad_()
    Wtt = torch.from_numpy(Wt).double().requires_grad_()
    bt = torch.from_numpy(b).double().requires_grad_()
    Yt = Fn.conv2d(Xt, Wtt, bt, stride=(sh, sw), padding=(ph, pw))
    Yt.backward(torch.from_numpy(dY).double())
    np.testing.assert_allclose(oracle.conv_forward(s, X, Wt, b), Yt.detach().numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(oracle.conv_backward_data(s, dY, Wt), Xt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(oracle.conv_backward_weights(s, X, dY), Wtt.grad.numpy(), rtol=0, atol=1e-10)
    np.testing.assert_allclose(oracle.bias_grad(s, dY), bt.grad.numpy(), rtol=0, atol=1e-10)


# ----------------------------------------------------------------------------- gradients

@pytest.mark.parametrize("cfg", TINY)
def test_adjoint_identities(cfg):
    # <conv(X,W), G> = <X, dgrad(G,W)> = <W, wgrad(X,G)>; <1 b, G> = <b, dbias(G)>.
    s, X, Wt, b, G = _mk(cfg, 80)
    lhs = np.sum(oracle.conv_forward(s, X, Wt) * G)
    assert np.isclose(lhs, np.sum(X * oracle.conv_backward_data(s, G, Wt)), rtol=1e-12, atol=1e-10)
    assert np.isclose(lhs, np.sum(Wt * oracle.conv_backward_weights(s, X, G)), rtol=1e-12, atol=1e-10)
    with_b = np.sum(oracle.conv_forward(s, X, Wt, b) * G)
    assert np.isclose(with_b - lhs, np.sum(b * oracle.bias_grad(s, G)), rtol=1e-10, atol=1e-9)


@pytest.mark.parametrize("cfg", TINY[:6])
def test_finite_differences(cfg):
    # l = <conv(X,W)+b, G> is bilinear, so a central difference is exact up to rounding.
    s, X, Wt, b, G = _mk(cfg, 100)
    X, Wt, b = np.round(X * 8) / 8, np.round(Wt * 8) / 8, np.round(b * 8) / 8   # exact in float32 +- h
    loss = lambda x, w, bb: np.sum(oracle.conv_forward(s, x, w, bb) * G)
    dX, dW, db = oracle.conv_backward_data(s, G, Wt), oracle.conv_backward_weights(s, X, G), oracle.bias_grad(s, G)
    rng = np.random.default_rng(7)
    h = 0.5
    for _ in range(6):
        i = tuple(rng.integers(0, d) for d in X.shape)
        e = np.zeros_like(X); e[i] = h
        assert np.isclose((loss(X + e, Wt, b) - loss(X - e, Wt, b)) / (2 * h), dX[i], rtol=1e-9, atol=1e-9)
        j = tuple(rng.integers(0, d) for d in Wt.shape)
        e = np.zeros_like(Wt); e[j] = h
        assert np.isclose((loss(X, Wt + e, b) - loss(X, Wt - e, b)) / (2 * h), dW[j], rtol=1e-9, atol=1e-9)
    e = np.zeros_like(b); e[0] = h
    assert np.isclose((loss(X, Wt, b + e) - loss(X, Wt, b - e)) / (2 * h), db[0], rtol=1e-9, atol=1e-9)


def test_gradients_sum_over_the_batch_without_scaling():
    # Sec. II-B: per-image gradients are summed; duplicating the batch doubles dW and dbias.
    s1, X, Wt, b, G = _mk((2, 2, 6, 6, 3, 3, 3, 1, 1, 1, 1), 120)
    s2 = oracle.shape(4, 2, 6, 6, 3, 3, 3, 1, 1)
    X2, G2 = np.concatenate([X, X]), np.concatenate([G, G])
    np.testing.assert_allclose(oracle.conv_backward_weights(s2, X2, G2), 2 * oracle.conv_backward_weights(s1, X, G), rtol=1e-13)
    np.testing.assert_allclose(oracle.bias_grad(s2, G2), 2 * oracle.bias_grad(s1, G), rtol=1e-13)


@pytest.mark.parametrize("cfg", TINY + [(2, 3, 23, 23, 4, 11, 11, 4, 4, 0, 0)])
def test_single_entry_routines_match_full_tensors(cfg):
    s, X, Wt, b, G = _mk(cfg, 140)
    Y, dX, dW = oracle.conv_forward(s, X, Wt, b), oracle.conv_backward_data(s, G, Wt), oracle.conv_backward_weights(s, X, G)
    for full, at in ((Y, lambda i: oracle.conv_forward_at(s, X, Wt, b, i)),
                     (dX, lambda i: oracle.conv_backward_data_at(s, G, Wt, i)),
                     (dW, lambda i: oracle.conv_backward_weights_at(s, X, G, i))):
        idx = np.arange(full.size)
        np.testing.assert_allclose(at(idx), full.ravel(), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- lowering / col2im

@pytest.mark.parametrize("cfg", TINY)
def test_lowering_is_a_copy_with_known_zero_count(cfg):
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
    ho, wo = oracle.out_dims(s)
    X = (np.arange(N * C * H * W, dtype=np.float32) + 1.0).reshape(N, C, H, W)   # no zeros, all distinct
    D = oracle.lower(s, X)
    assert D.shape == (C * kh * kw, N * ho * wo)
    assert np.array_equal(D, lr.lower(X, kh, kw, sh, sw, ph, pw))
    # torch's unfold is the same map per image: [N][C*kh*kw][Ho*Wo]
    U = Fn.unfold(torch.from_numpy(X), (kh, kw), padding=(ph, pw), stride=(sh, sw)).numpy()
    assert np.array_equal(D, U.transpose(1, 0, 2).reshape(C * kh * kw, -1))
    cy = sum(sum(0 <= oy * sh - ph + t < H for t in range(kh)) for oy in range(ho))
    cx = sum(sum(0 <= ox * sw - pw + t < W for t in range(kw)) for ox in range(wo))
    assert np.count_nonzero(D) == N * C * cy * cx          # closed-form count of in-image entries
    assert set(np.unique(D[D != 0])) <= set(X.ravel())


def test_replication_factor_matches_paper_formula():
    # App. C: size(D-hat)/size(D) = m^2 k^2 / n^2.
    assert _facts()["replication_formula"] == "m*m*k*k/(n*n)"
    expect = {"conv1": 55 ** 2 * 11 ** 2 / 227 ** 2, "conv2": 25.0, "conv3": 9.0, "conv4": 9.0, "conv5": 9.0}
    for L in wl.caffenet_stack(2):
        s = oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)
        ho, wo = oracle.out_dims(s)
        ratio = (L.C * L.k * L.k * L.N * ho * wo) / (L.N * L.C * L.H * L.W)
        assert np.isclose(ratio, expect[L.name])
        assert np.isclose(ratio, ho * ho * L.k * L.k / (L.H * L.H))
    assert abs(expect["conv1"] - 7.10) < 0.01
    L = wl.caffenet_stack(1)[2]
    s = oracle.shape(1, 4, L.H, L.W, 1, L.k, L.k, L.s, L.p)
    assert oracle.lower(s, np.ones((1, 4, 13, 13), np.float32)).size == 9 * 4 * 13 * 13


@pytest.mark.parametrize("cfg", TINY)
def test_col2im_is_the_transpose_of_lowering(cfg):
    N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
    ho, wo = oracle.out_dims(s)
    X = _rand((N, C, H, W), 160)
    Z = _rand((C * kh * kw, N * ho * wo), 161)
    assert np.isclose(np.sum(oracle.lower(s, X).astype(np.float64) * Z), np.sum(X * oracle.col2im(s, Z)), rtol=1e-12, atol=1e-10)
    np.testing.assert_allclose(oracle.col2im(s, Z), lr.col2im(Z.astype(np.float64), N, C, H, W, kh, kw, sh, sw, ph, pw), rtol=0, atol=1e-13)
    # library: torch fold sums the same entries
    Zt = torch.from_numpy(Z).double().reshape(C * kh * kw, N, ho * wo).permute(1, 0, 2)
    fold = Fn.fold(Zt, (H, W), (kh, kw), padding=(ph, pw), stride=(sh, sw)).numpy()
    np.testing.assert_allclose(oracle.col2im(s, Z), fold, rtol=0, atol=1e-12)
    # col2im(lower(X)) = X * multiplicity, multiplicity = per-axis counts of windows covering a pixel
    my = np.array([sum(1 for ky in range(kh) if (iy + ph - ky) >= 0 and (iy + ph - ky) % sh == 0 and (iy + ph - ky) // sh < ho) for iy in range(H)])
    mx = np.array([sum(1 for kx in range(kw) if (ix + pw - kx) >= 0 and (ix + pw - kx) % sw == 0 and (ix + pw - kx) // sw < wo) for ix in range(W)])
    np.testing.assert_allclose(oracle.col2im(s, oracle.lower(s, X)), X * np.outer(my, mx), rtol=1e-13)
    if sh == 1 and sw == 1 and ph == kh // 2 and pw == kw // 2 and H > 2 * kh and W > 2 * kw:
        assert my[kh] == kh and mx[kw] == kw               # k^2 in the interior


def test_matmul_against_numpy():
    A, B = _rand((7, 5), 1).astype(np.float64), _rand((5, 9), 2).astype(np.float64)
    np.testing.assert_allclose(oracle.matmul(A, B), A @ B, rtol=1e-14)
    assert np.array_equal(oracle.matmul(np.eye(5), B), B)
    # not symmetric in its operands: catches a transposed operand
    assert not np.allclose(oracle.matmul(A[:5, :5], B[:, :5]), oracle.matmul(B[:, :5], A[:5, :5]))


# ----------------------------------------------------------------------------- work accounting

def test_flop_rule_reproduces_the_papers_1p6_tflop():
    # Sec. II-C / App. B: conv1..5 at batch 256, three GEMMs per layer, conv1's data gradient skipped.
    facts = _facts()
    layers = wl.caffenet_stack(int(facts["alexnet_batch"]))
    per = [oracle.conv_flops(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p) for L in layers]
    assert per == [L.gemm_flops for L in layers]
    total = 3 * sum(per) - per[0]
    assert round(total / 1e12, 1) == float(facts["alexnet_conv_tflop_per_iteration"])
    assert abs(total / 1e9 - 1599.7) < 0.1
    assert abs(sum(per) / 1e9 - 551.2) < 0.1
    ks, ns, ds = [L.k for L in layers], [L.H for L in layers], [L.C for L in layers]
    assert (min(ks), max(ks)) == (int(facts["alexnet_k_min"]), int(facts["alexnet_k_max"]))
    assert (min(ns), max(ns)) == (int(facts["alexnet_n_min"]), int(facts["alexnet_n_max"]))
    assert (min(ds), max(ds)) == (int(facts["alexnet_din_min"]), int(facts["alexnet_din_max"]))
    assert wl.cifar_stack()[0].N == int(facts["batch_cifar"])


# ----------------------------------------------------------------------------- update

def test_sgd_closed_forms():
    rng = np.random.default_rng(3)
    W0 = rng.standard_normal(50).astype(np.float32)
    G = rng.standard_normal(50).astype(np.float32)
    Z = np.zeros(50, np.float32)
    W64, G64 = W0.astype(np.float64), G.astype(np.float64)
    # mu = 0, lambda = 0: plain gradient step
    W1, V1 = oracle.sgd_momentum(W0, Z, G, 0.1, 0.0, 0.0)
    np.testing.assert_allclose(W1, W64 - 0.1 * G64, rtol=1e-15)
    np.testing.assert_allclose(V1, -0.1 * G64, rtol=1e-15)
    # first step from V = 0 with lr 0.01, mu 0.9: V = -0.01 G (sign of V is observable)
    _, V1 = oracle.sgd_momentum(W0, Z, G, 0.01, 0.9, 0.0)
    np.testing.assert_allclose(V1, -0.01 * G64, rtol=1e-15)
    # constant gradient: geometric series for V and W (iterate in float64 through float32-exact values)
    eta, mu, T = 0.5, 0.5, 6
    Gc = np.full(4, 2.0, np.float32)
    Wc, Vc = np.zeros(4, np.float32), np.zeros(4, np.float32)
    for t in range(1, T + 1):
        Wn, Vn = oracle.sgd_momentum(Wc, Vc, Gc, eta, mu, 0.0)
        Wc, Vc = Wn.astype(np.float32), Vn.astype(np.float32)
        assert np.array_equal(Wn, Wc) and np.array_equal(Vn, Vc)            # dyadic values: exact
        v_closed = -eta * 2.0 * (1 - mu ** t) / (1 - mu)
        w_closed = -eta * 2.0 * (t - mu * (1 - mu ** t) / (1 - mu)) / (1 - mu)
        assert np.allclose(Vn, v_closed, rtol=1e-15) and np.allclose(Wn, w_closed, rtol=1e-15)
    # G = 0, mu = 0: pure weight decay, W_t = W_0 (1 - eta lambda)^t; the lambda term uses the OLD W
    W1, V1 = oracle.sgd_momentum(W0, Z, Z, 0.25, 0.0, 0.5)
    np.testing.assert_allclose(W1, W64 * (1 - 0.125), rtol=1e-15)
    np.testing.assert_allclose(V1, -0.125 * W64, rtol=1e-15)
    # momentum alone carries the step: W1 = W0 + mu V0
    V0 = rng.standard_normal(50).astype(np.float32)
    W1, V1 = oracle.sgd_momentum(W0, V0, Z, 0.3, 0.9, 0.0)
    np.testing.assert_allclose(V1, 0.9 * V0.astype(np.float64), rtol=1e-15)
    np.testing.assert_allclose(W1, W64 + 0.9 * V0.astype(np.float64), rtol=1e-15)


# ----------------------------------------------------------------------------- glue layers

def test_relu():
    x = np.array([-2.0, -0.0, 0.0, 1e-30, 3.5], np.float32)
    assert np.array_equal(oracle.relu_forward(x), np.array([0, 0, 0, np.float32(1e-30), 3.5], np.float64))
    assert np.array_equal(oracle.relu_backward(x, np.full(5, 2.0, np.float32)), np.array([0, 0, 0, 2, 2], np.float64))


@pytest.mark.parametrize("H,W,ceil_mode", [(32, 32, True), (32, 32, False), (16, 16, True), (8, 8, True),
                                            (55, 55, False), (55, 55, True), (13, 13, True), (7, 9, True), (6, 5, False)])
def test_maxpool_against_brute_force_and_torch(H, W, ceil_mode):
    x = _rand((2, 3, H, W), 200)
    y, am = oracle.maxpool_forward(x, 3, 2, ceil_mode)
    yt, it = Fn.max_pool2d(torch.from_numpy(x), 3, 2, ceil_mode=ceil_mode, return_indices=True)
    assert y.shape == tuple(yt.shape)
    assert np.array_equal(y, yt.double().numpy())
    assert np.array_equal(am, it.numpy())                  # distinct random values: argmax is unique
    for (n, c, oy, ox) in [(0, 0, 0, 0), (1, 2, y.shape[2] - 1, y.shape[3] - 1), (1, 1, 1, y.shape[3] - 1)]:
        win = x[n, c, oy * 2:min(oy * 2 + 3, H), ox * 2:min(ox * 2 + 3, W)]
        assert y[n, c, oy, ox] == win.max()
    g = _rand(y.shape, 201)
    dx = oracle.maxpool_backward(g, am, H, W)
    xt = torch.from_numpy(x).double().requires_grad_()
    Fn.max_pool2d(xt, 3, 2, ceil_mode=ceil_mode).backward(torch.from_numpy(g).double())
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=0, atol=1e-15)


def test_maxpool_sizes_and_tie_rule():
    assert [oracle.pool_out_dim(n, 3, 2, True) for n in (32, 16, 8, 55, 27, 13)] == [16, 8, 4, 27, 13, 6]
    assert [oracle.pool_out_dim(n, 3, 2, False) for n in (32, 15, 7, 55, 27, 13)] == [15, 7, 3, 27, 13, 6]
    ramp = np.arange(49, dtype=np.float32).reshape(1, 1, 7, 7)
    y, am = oracle.maxpool_forward(ramp, 3, 2, False)
    assert np.array_equal(am[0, 0], np.array([[16, 18, 20], [30, 32, 34], [44, 46, 48]]))   # last element of each window
    const = np.full((1, 1, 7, 7), 2.0, np.float32)
    y, am = oracle.maxpool_forward(const, 3, 2, False)
    assert np.array_equal(am[0, 0], np.array([[0, 2, 4], [14, 16, 18], [28, 30, 32]]))      # first element wins ties
    dx = oracle.maxpool_backward(np.ones((1, 1, 3, 3), np.float32), am, 7, 7)
    assert dx.sum() == 9 and dx[0, 0, 0, 0] == 1 and dx[0, 0, 1, 1] == 0


# ----------------------------------------------------------------------------- workloads

def test_workload_generators_are_seeded_and_distributed_as_stated():
    L = wl.single_layer_config()
    a, b = wl.layer_tensors(L, seed=1, x_dist="uniform"), wl.layer_tensors(L, seed=1, x_dist="uniform")
    assert all(np.array_equal(a[k], b[k]) for k in a)
    c = wl.layer_tensors(L, seed=2, x_dist="uniform")
    assert not np.array_equal(a["X"], c["X"])
    assert a["X"].min() >= -1 and a["X"].max() < 1 and abs(a["X"].mean()) < 0.02
    assert abs(a["W"].std() - 0.01) < 0.001 and abs(a["dY"].std() - 1) < 0.01
    h = wl.layer_tensors(L, seed=1, bf16=True)
    assert np.array_equal(h["X"], wl.to_bf16_values(h["X"]))
    assert np.all((h["X"].view(np.uint32) & 0xFFFF) == 0)        # bf16-representable
    st = wl.stack_tensors(wl.cifar_stack(4), seed=1, x_dist="uniform", pooled_out=(4, 4))
    assert st["dY"].shape == (4, 64, 4, 4) and len(st["W"]) == 3


# ---------------------------------------------------------------- normalisation across channels
LRN_CASES = [(2, 7, 3, 4, 5, 1e-4, 0.75, 1.0), (1, 5, 2, 2, 3, 0.3, 0.5, 2.0), (2, 3, 1, 5, 5, 2.0, 0.75, 1.0),
             (1, 9, 3, 3, 1, 0.7, 1.0, 0.5), (1, 12, 2, 3, 7, 0.05, 0.75, 1.0)]


@pytest.mark.parametrize("N,C,H,W,size,alpha,beta,k", LRN_CASES)
def test_lrn_matches_the_library_routine_and_its_autograd(N, C, H, W, size, alpha, beta, k):
    x = _rand((N, C, H, W), 31) * 3.0
    g = _rand((N, C, H, W), 32)
    xt = torch.from_numpy(x.astype(np.float64)).requires_grad_(True)
    yt = Fn.local_response_norm(xt, size, alpha=alpha, beta=beta, k=k)
    yt.backward(torch.from_numpy(g.astype(np.float64)))
    np.testing.assert_allclose(oracle.lrn_forward(x, size, alpha, beta, k), yt.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.lrn_backward(x, g, size, alpha, beta, k), xt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_lrn_closed_forms():
    # constant input a: a full window holds `size` copies of a^2, so y = a / (k + alpha a^2)^beta in the
    # interior; the first and last channels see a window clipped to (size+1)/2 terms but still divide by size
    a, size, alpha, beta, k, C = 1.5, 5, 0.2, 0.75, 1.0, 9
    y = oracle.lrn_forward(np.full((2, C, 3, 3), a, dtype=np.float32), size, alpha, beta, k)
    np.testing.assert_allclose(y[:, 2:C - 2], a / (k + alpha * a * a) ** beta, rtol=1e-14)
    np.testing.assert_allclose(y[:, 0], a / (k + alpha / size * 3 * a * a) ** beta, rtol=1e-14)
    np.testing.assert_allclose(y[:, 1], a / (k + alpha / size * 4 * a * a) ** beta, rtol=1e-14)
    np.testing.assert_allclose(y[:, C - 1], y[:, 0], rtol=1e-15)
    # a window of one channel with beta = 1: y = x / (k + alpha x^2), dy/dx = (k - alpha x^2) / (k + alpha x^2)^2
    x = _rand((1, 4, 2, 3), 33) * 2.0
    x64 = x.astype(np.float64)
    np.testing.assert_allclose(oracle.lrn_forward(x, 1, 0.3, 1.0, 2.0), x64 / (2.0 + 0.3 * x64 ** 2), rtol=1e-14)
    np.testing.assert_allclose(oracle.lrn_backward(x, np.ones_like(x), 1, 0.3, 1.0, 2.0),
                               (2.0 - 0.3 * x64 ** 2) / (2.0 + 0.3 * x64 ** 2) ** 2, rtol=1e-12)
    # alpha = 0: a plain scaling by k^-beta in both directions
    np.testing.assert_allclose(oracle.lrn_forward(x, 5, 0.0, 0.75, 4.0), x64 * 4.0 ** -0.75, rtol=1e-14)
    np.testing.assert_allclose(oracle.lrn_backward(x, x, 5, 0.0, 0.75, 4.0), x64 * 4.0 ** -0.75, rtol=1e-14)
    with pytest.raises(ValueError):
        oracle.lrn_forward(x, 4)


def test_lrn_backward_by_central_differences():
    N, C, H, W, size, alpha, beta, k = 1, 6, 2, 2, 5, 0.5, 0.75, 1.0
    x = _rand((N, C, H, W), 34) * 2.0
    g = _rand((N, C, H, W), 35).astype(np.float64)
    dx = oracle.lrn_backward(x, g.astype(np.float32), size, alpha, beta, k)
    g = g.astype(np.float32).astype(np.float64)
    h = 2.0 ** -10                      # exactly representable steps of float32 inputs of this size
    for idx in itertools.product(range(N), range(C), range(H), range(W)):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        step = float(xp[idx]) - float(xm[idx])
        fd = np.sum(g * (oracle.lrn_forward(xp, size, alpha, beta, k) - oracle.lrn_forward(xm, size, alpha, beta, k))) / step
        assert abs(fd - dx[idx]) <= 1e-5 * max(1.0, abs(dx[idx])), (idx, fd, dx[idx])


# ---------------------------------------------------------------- dropout and its generator
def test_philox_blocks_match_numpys_generator():
    # numpy's Philox bit generator is the same Philox4x64-10; it advances its counter before it
    # produces a block, so its first four raw words are the block of counter + 1
    for ctr, key in (([0, 0, 0, 0], [0, 0]), ([5, 0, 0, 0], [1, 2]), ([2 ** 64 - 2, 7, 0, 3], [123456789, 42]),
                     ([41, 0, 0, 0], [2 ** 64 - 1, 2 ** 63])):
        bg = np.random.Philox(counter=np.array(ctr, dtype=np.uint64), key=np.array(key, dtype=np.uint64))
        nxt = list(ctr)
        nxt[0] += 1
        assert oracle.philox4x64(nxt, key) == [int(v) for v in bg.random_raw(4)]


def _numpy_draws(count, seed, stream):
    """The 32-bit draws of elements 0..count-1, taken from numpy's Philox: blocks 0, 1, 2, ... are what a
    generator started one counter step before zero produces (counter all ones wraps to zero)."""
    bg = np.random.Philox(counter=np.array([2 ** 64 - 1] * 4, dtype=np.uint64), key=np.array([seed, stream], dtype=np.uint64))
    raw = bg.random_raw(4 * ((count + 7) // 8))
    lo, hi = raw & np.uint64(0xffffffff), raw >> np.uint64(32)
    return np.stack([lo, hi], axis=1).reshape(-1)[:count]


@pytest.mark.parametrize("count,p,seed,stream", [(1000, 0.5, 1, 0), (37, 0.25, 7, 3), (4096, 0.9, 2 ** 40 + 5, 1), (8, 0.5, 0, 0)])
def test_dropout_mask_is_draw_at_least_threshold(count, p, seed, stream):
    draws = _numpy_draws(count, seed, stream)
    thr = int(np.floor(p * 2.0 ** 32))
    assert oracle.dropout_threshold(p) == thr
    keep = oracle.dropout_mask(count, p, seed, stream)
    assert np.array_equal(keep, (draws >= thr).astype(np.uint8))
    x = _rand((count,), 40)
    y = oracle.dropout_apply(x, p, seed, stream)
    np.testing.assert_allclose(y, np.where(keep == 1, x.astype(np.float64) / (1.0 - p), 0.0), rtol=1e-15)


def test_dropout_invariants():
    n, p = 1 << 16, 0.5
    x = _rand((n,), 41)
    g = _rand((n,), 42)
    keep = oracle.dropout_mask(n, p, 1)
    # kept fraction within five standard deviations of 1 - p
    assert abs(keep.mean() - (1 - p)) <= 5 * np.sqrt(p * (1 - p) / n)
    # p = 0 keeps everything unscaled; the threshold saturates below 2^32
    assert np.array_equal(oracle.dropout_apply(x, 0.0, 9), x.astype(np.float64))
    assert oracle.dropout_threshold(0.0) == 0 and oracle.dropout_threshold(1.0) == 2 ** 32 - 1
    # the map is diagonal, hence its own adjoint: <drop(x), g> = <x, drop(g)>
    np.testing.assert_allclose(np.dot(oracle.dropout_apply(x, p, 1), g.astype(np.float64)),
                               np.dot(x.astype(np.float64), oracle.dropout_apply(g, p, 1)), rtol=1e-12)
    # scaling keeps the expectation: mean of y ~ mean of x for a constant input
    y = oracle.dropout_apply(np.ones(n, dtype=np.float32), p, 1)
    assert abs(y.mean() - 1.0) <= 5 * np.sqrt(p / (1 - p) / n)
    # other seed or stream, other mask; same arguments, same mask
    assert not np.array_equal(keep, oracle.dropout_mask(n, p, 2))
    assert not np.array_equal(keep, oracle.dropout_mask(n, p, 1, 1))
    assert np.array_equal(keep, oracle.dropout_mask(n, p, 1))
    # a longer call extends a shorter one (element i depends on i, seed and stream only)
    assert np.array_equal(oracle.dropout_mask(1001, p, 1), keep[:1001])
