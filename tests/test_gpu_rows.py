"""GPU parity of the "rows" form of a layer's output gradient: the matrix [F][N * pitch] that the model gradient
multiplies, written directly by the layer that produces the gradient (ReLU backward, max-pool backward) and read
by both backward passes of the convolution.

The producers move values without arithmetic, so their outputs are compared exactly with the oracle's dense result
put into that layout (ReLU) or with the dense GPU pass that is itself checked against the oracle (pool); the
plane sums are fp32 sums in a fixed order and are compared with the fp64 sums of the same values.  The consumers run
the same kernels on the same values as the plain entry points, so dW and dX must be bit-identical to theirs, and
the bias gradient is compared with the oracle's.
"""
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


def gpu(a, bf16=True):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rows_of(dense, ld=None, fill=0.0):
    """[N][C][h][w] (numpy) -> the rows matrix [C][ld], planes rounded up to 8 elements with zeros."""
    N, C = dense.shape[:2]
    plane = dense.shape[2] * dense.shape[3]
    pitch = (plane + 7) // 8 * 8
    out = np.full((C, ld or N * pitch), fill, dtype=np.float64)
    block = np.zeros((C, N, pitch))
    block[:, :, :plane] = dense.reshape(N, C, plane).transpose(1, 0, 2)
    out[:, :N * pitch] = block.reshape(C, N * pitch)
    return out


def check_sums(sums, dense):
    ref = dense.sum(axis=(2, 3)).T                      # [C][N]
    scale = np.abs(dense).sum(axis=(2, 3)).T + 1e-30
    assert np.max(np.abs(host(sums) - ref) / scale) <= 1e-5


@pytest.mark.parametrize("N,C,h,w", [(3, 5, 13, 13), (16, 4, 27, 27), (2, 3, 2, 4), (300, 2, 3, 5), (1, 1, 32, 64),
                                      (23, 7, 13, 13), (5, 2, 9, 1)])
def test_relu_backward_rows(B, N, C, h, w):
    """Planes of whole and ragged 8-element packs, one to 128 images per workgroup with a ragged last group, the
    largest plane; every element of the matrix is written (it starts as NaN)."""
    print("relu rows", N, C, h, w, flush=True)
    rng = np.random.default_rng(N * 1000 + h * w)
    y = wl.to_bf16_values(np.maximum(rng.standard_normal((N, C, h, w)), 0.0))
    dy = wl.to_bf16_values(rng.standard_normal((N, C, h, w)))
    ref = oracle.relu_backward(y, dy)
    pitch = (h * w + 7) // 8 * 8
    out = torch.full((C, N * pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
    rows, sums = B.relu_backward_rows(gpu(y), gpu(dy), dx_rows=out)
    assert np.array_equal(host(rows), rows_of(ref))
    check_sums(sums, ref)
    # a longer leading dimension: the columns behind the last plane stay as they were; no sums wanted
    out = torch.full((C, N * pitch + 16), 7.0, dtype=torch.bfloat16, device="cuda")
    rows, none = B.relu_backward_rows(gpu(y), gpu(dy), dx_rows=out, ld=N * pitch + 16, want_sums=False)
    assert none is None and np.array_equal(host(rows), rows_of(ref, N * pitch + 16, 7.0))


def test_relu_backward_rows_declines(B):
    y = torch.zeros((1, 1, 1, 4), dtype=torch.bfloat16, device="cuda")          # plane of fewer than 8 elements
    with pytest.raises(B.OmniError):
        B.relu_backward_rows(y, y)
    y = torch.zeros((1, 1, 8, 8), dtype=torch.float32, device="cuda")           # fp32
    with pytest.raises(B.OmniError):
        B.relu_backward_rows(y, y, dx_rows=torch.zeros((1, 64), device="cuda"))


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("N,C,H,W,ceil_mode", [(2, 3, 13, 13, True), (4, 6, 27, 27, True), (1, 2, 55, 55, True),
                                                (3, 2, 12, 9, False), (5, 1, 7, 30, True), (37, 3, 13, 13, False),
                                                (2, 5, 8, 8, True)])
def test_maxpool_backward_rows(B, N, C, H, W, ceil_mode, relu):
    """3 x 3 / stride 2 pool backward (with and without the ReLU mask) into the rows matrix: equal to the dense pass,
    which is checked against the oracle here as well; zero round-ups; plane sums."""
    print("pool rows", N, C, H, W, ceil_mode, relu, flush=True)
    rng = np.random.default_rng(H * 100 + W + N)
    x = wl.to_bf16_values(np.round(rng.standard_normal((N, C, H, W)) * 2) / 2)    # many exact ties
    y_ref, am_ref = oracle.maxpool_forward(x, 3, 2, ceil_mode)
    yg, am = B.maxpool_forward(gpu(x), 3, 2, ceil_mode)
    dy = wl.to_bf16_values(rng.standard_normal(y_ref.shape))
    g_in = dy * (y_ref > 0) if relu else dy
    ref = oracle.maxpool_backward(g_in, am_ref, H, W)
    dense = B.maxpool_relu_backward(gpu(dy), am, yg, H, W, 3, 2, ceil_mode) if relu else \
        B.maxpool_backward(gpu(dy), am, H, W, 3, 2, ceil_mode)
    scale = np.max(np.abs(ref))
    assert np.max(np.abs(host(dense) - ref)) <= 2e-2 * scale
    pitch = (H * W + 7) // 8 * 8
    out = torch.full((C, N * pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
    rows, sums = B.maxpool_backward_rows(gpu(dy), am, yg if relu else None, H, W, 3, 2, ceil_mode, dx_rows=out)
    assert np.array_equal(host(rows), rows_of(host(dense)))
    check_sums(sums, host(dense))
    again, sums2 = B.maxpool_backward_rows(gpu(dy), am, yg if relu else None, H, W, 3, 2, ceil_mode)
    assert torch.equal(again, rows) and torch.equal(sums, sums2)


def test_maxpool_backward_rows_declines(B):
    dy = torch.zeros((1, 1, 2, 2), dtype=torch.bfloat16, device="cuda")
    am = torch.zeros((1, 1, 2, 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.OmniError):                                             # 2 x 2 windows
        B.maxpool_backward_rows(dy, am, None, 4, 4, 2, 2, True)


# (N, C, H, W, F, kh, kw, ph, pw), stride 1: layers whose model gradient reads the rows form
ROWS_SHAPES = [(4, 64, 13, 13, 128, 3, 3, 1, 1), (12, 64, 13, 13, 384, 3, 3, 1, 1), (8, 128, 13, 13, 256, 3, 3, 1, 1),
               (2, 96, 27, 27, 128, 5, 5, 2, 2), (4, 96, 8, 12, 256, 5, 5, 2, 2), (8, 96, 4, 15, 128, 7, 5, 3, 2)]


@pytest.mark.parametrize("cfg", ROWS_SHAPES)
def test_conv_backward_from_rows(B, cfg):
    """dY handed over as the rows matrix (written by relu_backward_rows from the dense gradient and a mask of ones
    and zeros): the model gradient and the data gradient are bit-identical to the plain entry points', the bias
    gradient matches the oracle, and dW matches the oracle too."""
    print("conv from rows", cfg, flush=True)
    N, C, H, W, F, kh, kw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (1, 1), (ph, pw))
    rng = np.random.default_rng(31)
    X = wl.to_bf16_values(rng.standard_normal((N, C, H, W)))
    Wt = wl.to_bf16_values(0.05 * rng.standard_normal((F, C, kh, kw)))
    dY = wl.to_bf16_values(rng.standard_normal((N, F, H, W)))
    mask = (rng.random((N, F, H, W)) < 0.6).astype(np.float64)
    d = B.conv_desc(N, C, H, W, F, kh, kw, (1, 1), (ph, pw), B.BF16, B.FLAG_FUSED)
    layout = B.conv_dy_rows_layout(d)
    assert layout is not None
    ld, pitch = layout
    assert pitch == (H * W + 7) // 8 * 8 and ld == N * pitch
    rows, sums = B.relu_backward_rows(gpu(mask), gpu(dY), ld=ld)
    dYm = dY * mask
    Xg, dYg, Wg = gpu(X), gpu(dYm), gpu(Wt)
    dW, db = B.conv_backward_weights_rows(d, Xg, rows, sums)
    dW_plain, db_plain = B.conv_backward_weights(d, Xg, dYg)
    assert torch.equal(dW, dW_plain)
    ref = oracle.conv_backward_weights(s, X, dYm)
    assert np.max(np.abs(host(dW) - ref)) <= 1e-4 * np.max(np.abs(ref))
    ref_b = oracle.bias_grad(s, dYm)
    assert np.max(np.abs(host(db) - ref_b)) <= 1e-4 * np.max(np.abs(ref_b))
    assert np.max(np.abs(host(db) - host(db_plain))) <= 1e-4 * np.max(np.abs(ref_b))
    dW2, none = B.conv_backward_weights_rows(d, Xg, rows, None, want_dbias=False)
    assert none is None and torch.equal(dW2, dW)
    nbytes = B.conv_packed_weights_bytes(d, B.PASS_BACKWARD_DATA)
    if nbytes:
        buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        B.conv_pack_weights([d], [B.PASS_BACKWARD_DATA], [Wg], [buf])
        dX = B.conv_backward_data_rows(d, rows, buf)
        assert torch.equal(dX, B.conv_backward_data_packed(d, dYg, buf))
        ref_x = oracle.conv_backward_data(s, dYm, Wt)
        assert np.max(np.abs(host(dX) - ref_x)) <= 2e-2 * np.max(np.abs(ref_x))
    else:
        with pytest.raises(B.OmniError):
            B.conv_backward_data_rows(d, rows, torch.empty(256, dtype=torch.uint8, device="cuda"))


def test_rows_layout_declines(B):
    # images x plane pitch not a multiple of 64, no fused flag, a strided layer: no rows form
    for cfg, flags, st in [((3, 64, 13, 13, 128, 3, 3, 1, 1), 4, 1), ((4, 64, 13, 13, 128, 3, 3, 1, 1), 0, 1),
                           ((4, 64, 13, 13, 128, 3, 3, 1, 1), 4, 2)]:
        N, C, H, W, F, kh, kw, ph, pw = cfg
        d = B.conv_desc(N, C, H, W, F, kh, kw, (st, st), (ph, pw), B.BF16, flags)
        assert B.conv_dy_rows_layout(d) is None


# (N, C, H, W, F, kh, kw, ph, pw) of the layer whose data gradient is taken, forced column tile (0: the library's
# choice); N large enough that the data gradient's reduction is not split over workgroups
RELU_ROWS_SHAPES = [((392, 64, 13, 13, 128, 3, 3, 1, 1), 0), ((392, 128, 13, 13, 128, 3, 3, 1, 1), 0),
                    ((96, 96, 27, 27, 128, 5, 5, 2, 2), 0), ((392, 192, 13, 13, 128, 3, 3, 1, 1), 0),
                    ((392, 128, 13, 13, 128, 3, 3, 1, 1), 256), ((392, 128, 13, 13, 128, 3, 3, 1, 1), 512),
                    ((392, 64, 13, 13, 128, 3, 3, 1, 1), 512)]


@pytest.mark.parametrize("cfg,bn", RELU_ROWS_SHAPES)
def test_conv_backward_data_relu_rows(B, cfg, bn):
    """The data gradient that stores (y_front > 0 ? dX : 0) as the front layer's rows matrix: bit-identical to the
    dense data gradient followed by relu_backward_rows; its column-tile sums add up to the rows' sums; the model
    gradient of the front layer takes them for its bias gradient.  Row tiles of 96 and 128 channels, a second row
    tile that is half empty, all three column tiles, pieces that straddle images, a ragged last column tile."""
    print("dgrad relu rows", cfg, bn, flush=True)
    N, C, H, W, F, kh, kw, ph, pw = cfg
    rng = np.random.default_rng(41)
    Wt = gpu(0.05 * rng.standard_normal((F, C, kh, kw)))
    dY = gpu(rng.standard_normal((N, F, H, W)))
    y_front = gpu(np.maximum(rng.standard_normal((N, C, H, W)), 0.0))
    d = B.conv_desc(N, C, H, W, F, kh, kw, (1, 1), (ph, pw), B.BF16, B.FLAG_FUSED)
    ld, pitch = B.conv_dy_rows_layout(d)
    rows, _ = B.relu_backward_rows(torch.ones_like(dY), dY, ld=ld)
    buf = torch.empty(B.conv_packed_weights_bytes(d, B.PASS_BACKWARD_DATA), dtype=torch.uint8, device="cuda")
    B.conv_pack_weights([d], [B.PASS_BACKWARD_DATA], [Wt], [buf])
    B.tuning_set(B.TUNE_FUSED_BN, bn)
    try:
        per = B.conv_backward_data_relu_rows_sums(d)
        assert per is not None and per >= 1
        dX = B.conv_backward_data_rows(d, rows, buf)
        got, sums = B.conv_backward_data_relu_rows(d, rows, buf, y_front)
        again, sums2 = B.conv_backward_data_relu_rows(d, rows, buf, y_front)
    finally:
        B.tuning_set(B.TUNE_FUSED_BN, 0)
    expect, plane_sums = B.relu_backward_rows(y_front, dX)
    assert torch.equal(got, expect)
    assert torch.equal(got, again) and torch.equal(sums, sums2)
    total = host(expect).sum(axis=1)
    scale = np.abs(host(expect)).sum(axis=1) + 1e-30
    assert np.max(np.abs(host(sums).sum(axis=1) - total) / scale) <= 1e-5
    assert tuple(sums.shape) == (C, per)
    if cfg == RELU_ROWS_SHAPES[1][0] and bn == 0:
        s = oracle.shape(N, C, H, W, F, kh, kw, (1, 1), (ph, pw))
        ref = oracle.conv_backward_data(s, host(dY), host(Wt)) * (host(y_front) > 0)
        assert np.max(np.abs(host(got) - rows_of(ref))) <= 2e-2 * np.max(np.abs(ref))
        # the front layer (a 3 x 3 layer of C filters on these planes) takes the column-tile sums for its bias gradient
        Cf = 64
        df = B.conv_desc(N, Cf, H, W, C, 3, 3, (1, 1), (1, 1), B.BF16, B.FLAG_FUSED)
        assert B.conv_dy_rows_layout(df) == (ld, pitch)
        Xf = gpu(rng.standard_normal((N, Cf, H, W)))
        dW_a, db_a = B.conv_backward_weights_rows(df, Xf, got, sums)
        dW_b, db_b = B.conv_backward_weights_rows(df, Xf, got, plane_sums)
        assert torch.equal(dW_a, dW_b)
        sf = oracle.shape(N, Cf, H, W, C, 3, 3, (1, 1), (1, 1))
        dense = host(got).reshape(C, N, pitch)[:, :, :H * W].transpose(1, 0, 2).reshape(N, C, H, W)
        ref_b = oracle.bias_grad(sf, dense)
        assert np.max(np.abs(host(db_a) - ref_b)) <= 1e-4 * np.max(np.abs(ref_b))
        assert np.max(np.abs(host(db_b) - ref_b)) <= 1e-4 * np.max(np.abs(ref_b))


def test_conv_backward_data_relu_rows_declines_split_reductions(B):
    """Few column tiles (a small batch): the data gradient splits its reduction and cannot store the masked rows."""
    d = B.conv_desc(4, 64, 13, 13, 128, 3, 3, (1, 1), (1, 1), B.BF16, B.FLAG_FUSED)
    assert B.conv_dy_rows_layout(d) is not None
    assert B.conv_backward_data_relu_rows_sums(d) is None
