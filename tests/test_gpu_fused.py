"""GPU parity of the fused path (OMNI_FLAG_FUSED): forward and data gradient without D-hat in memory.

Same bar as the explicit path: bf16 storage, tensor-normalised error <= 2e-2 against the fp64 oracle on
identical bf16-representable inputs; and, because both paths add the same products in fp32 (in a
different order), the two GPU paths must agree with each other far more tightly than with the oracle's
tolerance.  Shapes cover several column tiles with a ragged last one, tiles that straddle images, a
second (nearly empty) row tile, non-square images and windows, padding 0 .. k-1, a 1 x 1 window, and
shapes the fused kernel must decline (stride 2, channels not a multiple of 32, fp32).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_04487_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-2
BF16 = 1


@pytest.fixture(scope="module")
def B():
    from paper_1606_04487_amd import binding
    assert torch.cuda.is_available()
    return binding


@pytest.fixture
def tuning(B):
    """Sets tile overrides through omni_tuning_set and puts the library's own choice back afterwards."""
    touched = []

    def set_knob(knob, value):
        touched.append(knob)
        B.tuning_set(knob, value)

    yield set_knob
    for knob in touched:
        B.tuning_set(knob, -1 if knob == B.TUNE_GEMM_TILE else 0)


def gpu(a, bf16=True):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    scale = np.max(np.abs(ref))
    return np.max(np.abs(got - ref)) / (scale if scale > 0 else 1.0)


# (N, C, H, W, F, kh, kw, ph, pw), stride 1
FUSED_SHAPES = [
    (6, 32, 13, 13, 40, 3, 3, 1, 1),      # tiles straddle images; F = 40
    (3, 64, 27, 27, 130, 5, 5, 2, 2),     # conv2-like; F = 130: second row tile nearly empty
    (20, 32, 8, 8, 64, 5, 5, 2, 2),       # CIFAR conv3-like: four images per tile
    (3, 32, 9, 11, 32, 3, 2, 0, 1),       # non-square image and window, no vertical padding
    (2, 64, 7, 5, 32, 3, 3, 2, 2),        # padding k - 1 (the data gradient then has none)
    (5, 32, 6, 6, 8, 1, 1, 0, 0),         # 1 x 1 window
    (1, 32, 3, 3, 8, 3, 3, 1, 1),         # a single 9-pixel image
    (2, 96, 27, 27, 256, 5, 5, 2, 2),     # conv2 at its real channel counts
    (4, 256, 13, 13, 384, 3, 3, 1, 1),    # conv3 at its real channel counts (F = 384: three 128-row tiles)
]


def make(cfg, seed):
    N, C, H, W, F, kh, kw, ph, pw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (1, 1), (ph, pw))
    ho, wo = oracle.out_dims(s)
    rng = np.random.default_rng(seed)
    X = wl.to_bf16_values(rng.standard_normal((N, C, H, W)))
    Wt = wl.to_bf16_values(0.05 * rng.standard_normal((F, C, kh, kw)))
    b = (0.05 * rng.standard_normal(F)).astype(np.float32)
    dY = wl.to_bf16_values(rng.standard_normal((N, F, ho, wo)))
    return s, X, Wt, b, dY


def desc_of(B, cfg, flags):
    N, C, H, W, F, kh, kw, ph, pw = cfg
    return B.conv_desc(N, C, H, W, F, kh, kw, (1, 1), (ph, pw), BF16, flags)


@pytest.mark.parametrize("cfg", FUSED_SHAPES)
def test_fused_forward(B, cfg):
    s, X, Wt, b, _ = make(cfg, 11)
    d = desc_of(B, cfg, B.FLAG_FUSED)
    assert B.conv_fused_supported(d, B.PASS_FORWARD)
    Xg, Wg, bg = gpu(X), gpu(Wt), gpu(b, False)
    ref = oracle.conv_forward(s, X, Wt, b)
    got = host(B.conv_forward(d, Xg, Wg, bg))
    assert rel_err(got, ref) <= TOL
    explicit = host(B.conv_forward(desc_of(B, cfg, 0), Xg, Wg, bg))
    assert rel_err(got, explicit) <= 1e-2          # one bf16 rounding step apart at most
    assert np.mean(got == explicit) > 0.9          # and nearly always the same rounding
    got_nb = host(B.conv_forward(d, Xg, Wg, None))
    assert rel_err(got_nb, oracle.conv_forward(s, X, Wt, None)) <= TOL
    got_relu = host(B.conv_forward(desc_of(B, cfg, B.FLAG_FUSED | B.FLAG_RELU), Xg, Wg, bg))
    assert rel_err(got_relu, np.maximum(ref, 0)) <= TOL and got_relu.min() >= 0
    again = host(B.conv_forward(d, Xg, Wg, bg))
    assert np.array_equal(got, again)              # deterministic


@pytest.mark.parametrize("cfg", FUSED_SHAPES)
def test_fused_backward_data(B, cfg):
    N, C, H, W, F, kh, kw, ph, pw = cfg
    if F % 32 != 0:
        # the data gradient reduces over F: declined, and the flag must fall back to the explicit path
        d = desc_of(B, cfg, B.FLAG_FUSED)
        assert not B.conv_fused_supported(d, B.PASS_BACKWARD_DATA)
    s, X, Wt, b, dY = make(cfg, 12)
    d = desc_of(B, cfg, B.FLAG_FUSED)
    dYg, Wg = gpu(dY), gpu(Wt)
    ref = oracle.conv_backward_data(s, dY, Wt)
    got = host(B.conv_backward_data(d, dYg, Wg))
    assert rel_err(got, ref) <= TOL
    explicit = host(B.conv_backward_data(desc_of(B, cfg, 0), dYg, Wg))
    assert rel_err(got, explicit) <= 1e-2
    again = host(B.conv_backward_data(d, dYg, Wg))
    assert np.array_equal(got, again)


@pytest.mark.parametrize("bn", ["256", "384", "512"])
@pytest.mark.parametrize("cfg", [FUSED_SHAPES[1], FUSED_SHAPES[2], FUSED_SHAPES[8], (7, 64, 13, 13, 96, 3, 3, 1, 1)])
def test_fused_every_column_tile(B, cfg, bn, tuning):
    """Each of the kernel's column-tile widths, forced through the tuning override, on both fused passes
    (a width whose patch does not fit a shape is skipped by the library, which then declines)."""
    tuning(B.TUNE_FUSED_BN, int(bn))
    s, X, Wt, b, dY = make(cfg, 21)
    d = desc_of(B, cfg, B.FLAG_FUSED | B.FLAG_RELU)
    ran = 0
    if B.conv_fused_supported(d, B.PASS_FORWARD):
        got = host(B.conv_forward(d, gpu(X), gpu(Wt), gpu(b, False)))
        assert rel_err(got, np.maximum(oracle.conv_forward(s, X, Wt, b), 0)) <= TOL
        ran += 1
    if B.conv_fused_supported(d, B.PASS_BACKWARD_DATA):
        got = host(B.conv_backward_data(d, gpu(dY), gpu(Wt)))
        assert rel_err(got, oracle.conv_backward_data(s, dY, Wt)) <= TOL
        ran += 1
    assert ran > 0 or bn != "256"


@pytest.mark.parametrize("bare", [0, 1])
@pytest.mark.parametrize("cfg", [FUSED_SHAPES[0], FUSED_SHAPES[1], (5, 96, 27, 27, 64, 5, 5, 2, 2), (9, 64, 13, 13, 128, 3, 3, 1, 1),
                                 (3, 32, 20, 22, 96, 3, 4, 1, 1)])
def test_fused_patch_pitch(B, cfg, bare, tuning):
    """The LDS patch with the bare padded row width and with the pitch that keeps fragment reads free of bank
    conflicts: the same sums in the same order, so the two agree bit for bit, and both meet the oracle."""
    print("fused patch pitch", cfg, "bare" if bare else "conflict-free", flush=True)
    s, X, Wt, b, dY = make(cfg, 29)
    d = desc_of(B, cfg, B.FLAG_FUSED | B.FLAG_RELU)
    tuning(B.TUNE_FUSED_PITCH, bare)
    Y = B.conv_forward(d, gpu(X), gpu(Wt), torch.from_numpy(b).cuda())
    assert rel_err(host(Y), np.maximum(oracle.conv_forward(s, X, Wt, b), 0.0)) <= TOL
    tuning(B.TUNE_FUSED_PITCH, 1 - bare)
    assert torch.equal(Y, B.conv_forward(d, gpu(X), gpu(Wt), torch.from_numpy(b).cuda()))
    if B.conv_fused_supported(d, B.PASS_BACKWARD_DATA):
        tuning(B.TUNE_FUSED_PITCH, bare)
        dX = B.conv_backward_data(d, gpu(dY), gpu(Wt))
        assert rel_err(host(dX), oracle.conv_backward_data(s, dY, Wt)) <= TOL
        tuning(B.TUNE_FUSED_PITCH, 1 - bare)
        assert torch.equal(dX, B.conv_backward_data(d, gpu(dY), gpu(Wt)))


@pytest.mark.parametrize("cfg", FUSED_SHAPES + [(3, 5, 13, 13, 7, 3, 3, 1, 1), (2, 20, 27, 27, 130, 5, 5, 2, 2),
                                                (2, 3, 9, 30, 4, 3, 5, 2, 4), (2, 30, 13, 13, 250, 3, 3, 1, 1),
                                                (3, 29, 9, 11, 256, 3, 2, 0, 1), (1, 57, 27, 27, 200, 5, 5, 2, 2),
                                                (2, 16, 20, 22, 256, 3, 4, 1, 1),    # rows of 3 packs
                                                (2, 8, 30, 28, 256, 3, 5, 1, 1),     # rows of 4 packs, Wo != W
                                                (3, 16, 9, 9, 384, 3, 3, 1, 1),      # 384-row tile, planes
                                                (2, 8, 60, 60, 256, 3, 3, 1, 1),     # plane too long for the mask table
                                                (1, 8, 3, 3, 256, 3, 3, 1, 1)])      # X barely larger than a pack
def test_fused_backward_weights(B, cfg):
    """Model gradient with the lowered operand read straight from X: the same products as the explicit
    path, summed in fp32 in another order (row-padded columns), within the fp32-output bar of the oracle."""
    N, C, H, W, F, kh, kw, ph, pw = cfg
    s, X, Wt, b, dY = make(cfg, 13)
    d = desc_of(B, cfg, B.FLAG_FUSED)
    wo = W + 2 * pw - kw + 1
    Xg, dYg = gpu(X), gpu(dY)
    dW, db = B.conv_backward_weights(d, Xg, dYg)
    assert rel_err(host(dW), oracle.conv_backward_weights(s, X, dY)) <= 1e-4
    assert rel_err(host(db), oracle.bias_grad(s, dY)) <= 1e-4
    dW2, _ = B.conv_backward_weights(desc_of(B, cfg, 0), Xg, dYg)
    assert rel_err(host(dW), host(dW2)) <= 2e-5
    again, _ = B.conv_backward_weights(d, Xg, dYg)
    assert torch.equal(dW, again)                  # deterministic


# 3 x 3 layers on 13 x 13 planes whose channels fill the LDS-patch model gradient's 128 x 64 tiles
PATCH_SHAPES = [(1, 64, 13, 13, 128, 3, 3, 1, 1), (2, 64, 13, 13, 128, 3, 3, 1, 1), (7, 128, 13, 13, 256, 3, 3, 1, 1),
                (12, 64, 13, 13, 384, 3, 3, 1, 1), (5, 192, 13, 13, 128, 3, 3, 1, 1)]


@pytest.mark.parametrize("splits", [0, 1, 2, 3])
@pytest.mark.parametrize("cfg", PATCH_SHAPES)
def test_patch_backward_weights(B, cfg, splits, tuning):
    """Model gradient with the lowered operand read from an LDS copy of the input planes: image ranges of one
    image, of whole pairs and with an odd last image (splits caps the number of ranges, so one workgroup walks
    several images), against the oracle and against the direct-loader path; deterministic."""
    print("patch wgrad", cfg, "splits", splits, flush=True)
    s, X, Wt, b, dY = make(cfg, 17)
    d = desc_of(B, cfg, B.FLAG_FUSED)
    tuning(B.TUNE_WGRAD_SPLITS, splits)
    Xg, dYg = gpu(X), gpu(dY)
    dW, db = B.conv_backward_weights(d, Xg, dYg)
    ref = oracle.conv_backward_weights(s, X, dY)
    assert rel_err(host(dW), ref) <= 1e-4
    assert rel_err(host(db), oracle.bias_grad(s, dY)) <= 1e-4
    again, _ = B.conv_backward_weights(d, Xg, dYg)
    assert torch.equal(dW, again)
    tuning(B.TUNE_WGRAD_PATCH, 1)                  # the same layer through the direct loader
    dW2, _ = B.conv_backward_weights(d, Xg, dYg)
    assert rel_err(host(dW), host(dW2)) <= 2e-5
    # every tap of every (filter, channel) pair is held to the bar on its own, so that a wrong mask or shift of
    # one tap cannot hide behind the tensor's maximum
    got = host(dW)
    for ky in range(3):
        for kx in range(3):
            assert rel_err(got[:, :, ky, kx], ref[:, :, ky, kx]) <= 1e-4, (ky, kx)


def test_packed_weights_entry_points_are_identical(B):
    """The caller-owned repacked weights: nine layer-and-pass pairs written by ONE launch, then the *_packed entry
    points against the plain ones, bit for bit (stride-1 layers both passes, the stride-4 layer forward)."""
    cfgs = [(3, 32, 13, 13, 64, 3, 3, 1, 1, 1), (2, 96, 27, 27, 256, 5, 5, 2, 2, 1), (5, 64, 13, 13, 384, 3, 3, 1, 1, 1),
            (2, 64, 9, 11, 128, 3, 2, 0, 1, 1), (2, 3, 67, 67, 96, 11, 11, 0, 0, 4)]
    rng = np.random.default_rng(23)
    jobs, cases = [], []
    for (N, C, H, W, F, kh, kw, ph, pw, st) in cfgs:
        d = B.conv_desc(N, C, H, W, F, kh, kw, st, (ph, pw), B.BF16, B.FLAG_FUSED | B.FLAG_RELU)
        ho, wo = B.conv_output_dims(d)
        X = gpu(rng.standard_normal((N, C, H, W)))
        Wt = gpu(0.05 * rng.standard_normal((F, C, kh, kw)))
        bias = torch.from_numpy(rng.standard_normal(F).astype(np.float32)).cuda()
        dY = gpu(rng.standard_normal((N, F, ho, wo)))
        for which in (B.PASS_FORWARD, B.PASS_BACKWARD_DATA):
            nbytes = B.conv_packed_weights_bytes(d, which)
            if nbytes == 0:
                assert st == 4 and which == B.PASS_BACKWARD_DATA
                continue
            buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            jobs.append((d, which, Wt, buf))
            cases.append((d, which, X, Wt, bias, dY, buf))
    assert len(jobs) == 9
    print("packed weights:", len(jobs), "jobs in one launch", flush=True)
    B.conv_pack_weights(*zip(*jobs))
    for d, which, X, Wt, bias, dY, buf in cases:
        print("packed entry point", d.N, d.C, d.H, d.F, d.kh, "pass", which, flush=True)
        if which == B.PASS_FORWARD:
            assert torch.equal(B.conv_forward_packed(d, X, buf, bias), B.conv_forward(d, X, Wt, bias))
        else:
            assert torch.equal(B.conv_backward_data_packed(d, dY, buf), B.conv_backward_data(d, dY, Wt))


# 5-wide windows, same-size output, channels a multiple of 96, filters of 128, planes of whole 32-position slabs:
# the LDS-patch model gradient with one window row per workgroup
WIDE_SHAPES = [(2, 96, 27, 27, 128, 5, 5, 2, 2), (3, 96, 8, 12, 256, 5, 5, 2, 2), (1, 192, 16, 16, 128, 5, 5, 2, 2),
               (2, 96, 12, 8, 128, 3, 5, 1, 2), (5, 96, 4, 15, 128, 7, 5, 3, 2), (1, 96, 24, 32, 128, 5, 5, 2, 2)]


@pytest.mark.parametrize("splits", [0, 1, 3])
@pytest.mark.parametrize("cfg", WIDE_SHAPES)
def test_wide_patch_backward_weights(B, cfg, splits, tuning):
    """Model gradient of 5-wide windows from LDS copies of plane windows (row offsets of every residue mod 8, window
    heights 3 to 7, planes with and without a ragged last group, two channel tiles, last stages of fewer slabs; one
    range of stages, three, or one round of workgroups), against the oracle tap by tap and against the direct-loader
    path; the bias gradient; deterministic."""
    print("wide patch wgrad", cfg, "splits", splits, flush=True)
    N, C, H, W, F, kh, kw, ph, pw = cfg
    s, X, Wt, b, dY = make(cfg, 19)
    d = desc_of(B, cfg, B.FLAG_FUSED)
    tuning(B.TUNE_WGRAD_SPLITS, splits)
    Xg, dYg = gpu(X), gpu(dY)
    dW, db = B.conv_backward_weights(d, Xg, dYg)
    ref = oracle.conv_backward_weights(s, X, dY)
    got = host(dW)
    assert rel_err(got, ref) <= 1e-4
    assert rel_err(host(db), oracle.bias_grad(s, dY)) <= 1e-4
    scale = np.max(np.abs(ref))
    for ky in range(kh):
        for kx in range(kw):
            assert np.max(np.abs(got[:, :, ky, kx] - ref[:, :, ky, kx])) <= 1e-4 * scale, (ky, kx)
    again, _ = B.conv_backward_weights(d, Xg, dYg)
    assert torch.equal(dW, again)
    tuning(B.TUNE_WGRAD_PATCH, 1)                  # the same layer without this kernel
    dW2, _ = B.conv_backward_weights(d, Xg, dYg)
    assert rel_err(got, host(dW2)) <= 2e-5


def test_fused_declines_and_falls_back(B):
    # stride 2, channels not a multiple of 32, fp32: the flag is accepted and the explicit path runs
    for cfg, dtype in [((2, 32, 9, 9, 8, 3, 3, 2, 2, 1, 1), 1), ((2, 20, 9, 9, 8, 3, 3, 1, 1, 1, 1), 1),
                       ((2, 32, 9, 9, 8, 3, 3, 1, 1, 1, 1), 0)]:
        N, C, H, W, F, kh, kw, sh, sw, ph, pw = cfg
        d = B.conv_desc(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw), dtype, B.FLAG_FUSED)
        assert not B.conv_fused_supported(d, B.PASS_FORWARD)
        if dtype != 1 or sh != 1:
            assert not B.conv_fused_supported(d, B.PASS_BACKWARD_WEIGHTS)
        s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (ph, pw))
        rng = np.random.default_rng(3)
        X = rng.standard_normal((N, C, H, W))
        Wt = 0.05 * rng.standard_normal((F, C, kh, kw))
        if dtype == 1:
            X, Wt = wl.to_bf16_values(X), wl.to_bf16_values(Wt)
        else:
            X, Wt = X.astype(np.float32), Wt.astype(np.float32)
        got = host(B.conv_forward(d, gpu(X, dtype == 1), gpu(Wt, dtype == 1), None))
        assert rel_err(got, oracle.conv_forward(s, X, Wt, None)) <= (TOL if dtype == 1 else 1e-4)


@pytest.mark.parametrize("cfg", [(3, 64, 27, 27, 48, 5, 5, 2, 2), (6, 32, 13, 13, 40, 3, 3, 1, 1),
                                 (2, 96, 27, 27, 96, 5, 5, 2, 2), (5, 32, 6, 6, 8, 1, 1, 0, 0)])
@pytest.mark.parametrize("bm", ["96", "128"])
def test_fused_row_tiles(B, cfg, bm, tuning):
    """Layers of few filters: the 96-row tile (forced up to 96 filters) and the 128-row tile agree with the oracle."""
    tuning(B.TUNE_FUSED_BM, int(bm))
    s, X, Wt, b, dY = make(cfg, 29)
    d = desc_of(B, cfg, B.FLAG_FUSED | B.FLAG_RELU)
    assert B.conv_fused_supported(d, B.PASS_FORWARD)
    got = host(B.conv_forward(d, gpu(X), gpu(Wt), gpu(b, False)))
    assert rel_err(got, np.maximum(oracle.conv_forward(s, X, Wt, b), 0)) <= TOL


# (N, C, H, W, F, kh, kw, sh): horizontal stride 4, no padding, few channels -- the conv1 kernel
STRIDED_SHAPES = [
    (2, 3, 35, 35, 8, 11, 11, 4),        # one tile per image, most of it beyond the image's last position
    (3, 3, 227, 227, 96, 11, 11, 4),     # conv1 itself: six tiles per image, ragged last one, 25 reduction steps
    (2, 2, 30, 41, 5, 3, 5, 2),          # window row of 5: the second group of 4 has one real column
    (1, 1, 12, 9, 3, 2, 1, 1),           # 1-wide window, vertical stride 1, a single channel
    (3, 4, 19, 23, 7, 4, 4, 3),          # window row of exactly one group
    (5, 3, 99, 99, 64, 7, 7, 4),         # 576 positions: a full tile and a short one
    (2, 3, 67, 131, 96, 11, 11, 4),      # non-square image
]


@pytest.mark.parametrize("cfg", STRIDED_SHAPES)
def test_strided_forward(B, cfg):
    N, C, H, W, F, kh, kw, sh = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, 4), (0, 0))
    rng = np.random.default_rng(17)
    X = wl.to_bf16_values(rng.standard_normal((N, C, H, W)))
    Wt = wl.to_bf16_values(0.05 * rng.standard_normal((F, C, kh, kw)))
    b = (0.05 * rng.standard_normal(F)).astype(np.float32)
    d = B.conv_desc(N, C, H, W, F, kh, kw, (sh, 4), (0, 0), BF16, B.FLAG_FUSED)
    assert B.conv_fused_supported(d, B.PASS_FORWARD)
    Xg, Wg, bg = gpu(X), gpu(Wt), gpu(b, False)
    ref = oracle.conv_forward(s, X, Wt, b)
    got = host(B.conv_forward(d, Xg, Wg, bg))
    assert rel_err(got, ref) <= TOL
    explicit = host(B.conv_forward(d.with_flags(0), Xg, Wg, bg))
    assert rel_err(got, explicit) <= 1e-2          # one bf16 rounding step apart at most
    assert np.mean(got == explicit) > 0.9
    got_relu = host(B.conv_forward(d.with_flags(B.FLAG_FUSED | B.FLAG_RELU), Xg, Wg, None))
    assert rel_err(got_relu, np.maximum(oracle.conv_forward(s, X, Wt, None), 0)) <= TOL and got_relu.min() >= 0
    assert np.array_equal(got, host(B.conv_forward(d, Xg, Wg, bg)))   # deterministic
    # pixels that only padded window columns reach never enter a sum: poison one of them
    if kw % 4 != 0 and W > kw:
        Xp = X.copy()
        Xp[:, :, :, kw] = np.inf                   # column kw: the first window's first padded column
        gotp = host(B.conv_forward(d, gpu(Xp), Wg, bg))
        assert np.array_equal(gotp[:, :, :, 0], got[:, :, :, 0])


@pytest.mark.parametrize("cfg", STRIDED_SHAPES + [(2, 3, 40, 239, 96, 11, 11, 4),   # Wo = 58: the last pack of a row runs past X4's row
                                                  (1, 16, 12, 45, 20, 2, 5, 3)])    # 16 channels, K' = 256
def test_strided_backward_weights(B, cfg):
    """Model gradient of a stride-4 layer from the four phase images of X (no D-hat): within the fp32-output
    bar of the oracle, close to the explicit path, deterministic; window columns beyond kw are dropped."""
    N, C, H, W, F, kh, kw, sh = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, 4), (0, 0))
    ho, wo = oracle.out_dims(s)
    rng = np.random.default_rng(19)
    X = wl.to_bf16_values(rng.standard_normal((N, C, H, W)))
    dY = wl.to_bf16_values(rng.standard_normal((N, F, ho, wo)))
    d = B.conv_desc(N, C, H, W, F, kh, kw, (sh, 4), (0, 0), BF16, B.FLAG_FUSED)
    # output rows shorter than a pack of 8 are left to the explicit path
    assert B.conv_fused_supported(d, B.PASS_BACKWARD_WEIGHTS) == (wo >= 8)
    Xg, dYg = gpu(X), gpu(dY)
    dW, db = B.conv_backward_weights(d, Xg, dYg)
    assert rel_err(host(dW), oracle.conv_backward_weights(s, X, dY)) <= 1e-4
    assert rel_err(host(db), oracle.bias_grad(s, dY)) <= 1e-4
    dW2, _ = B.conv_backward_weights(d.with_flags(0), Xg, dYg)
    assert rel_err(host(dW), host(dW2)) <= 2e-5
    again, db2 = B.conv_backward_weights(d, Xg, dYg)
    assert torch.equal(dW, again) and torch.equal(db, db2)   # deterministic


# (N, C, H, W, F, kh, kw, sh, sw): strided, unpadded layers whose data gradient runs as one stride-1 convolution
DGRAD_SHAPES = [
    (3, 3, 227, 227, 96, 11, 11, 4, 4),   # conv1
    (5, 3, 99, 99, 64, 7, 7, 4, 4),
    (2, 3, 67, 131, 96, 11, 11, 4, 4),    # non-square
    (2, 8, 21, 25, 32, 3, 5, 2, 4),       # different strides, window not a multiple of either
    (3, 16, 30, 30, 64, 5, 5, 2, 2),      # stride 2; the last input row and column are reached by no window
    (2, 4, 31, 33, 32, 3, 3, 4, 5),       # strides beyond the window: some phases have no tap at all
    (1, 2, 20, 23, 32, 4, 4, 3, 3),
    (2, 3, 35, 35, 40, 11, 11, 4, 4),     # F = 40: not a multiple of 32, the explicit path runs
]


@pytest.mark.parametrize("cfg", DGRAD_SHAPES)
def test_strided_backward_data(B, cfg):
    N, C, H, W, F, kh, kw, sh, sw = cfg
    s = oracle.shape(N, C, H, W, F, kh, kw, (sh, sw), (0, 0))
    ho, wo = oracle.out_dims(s)
    rng = np.random.default_rng(23)
    Wt = wl.to_bf16_values(0.05 * rng.standard_normal((F, C, kh, kw)))
    dY = wl.to_bf16_values(rng.standard_normal((N, F, ho, wo)))
    d = B.conv_desc(N, C, H, W, F, kh, kw, (sh, sw), (0, 0), BF16, B.FLAG_FUSED)
    assert B.conv_fused_supported(d, B.PASS_BACKWARD_DATA) == (F % 32 == 0)
    Wg, dYg = gpu(Wt), gpu(dY)
    ref = oracle.conv_backward_data(s, dY, Wt)
    got = host(B.conv_backward_data(d, dYg, Wg))
    assert rel_err(got, ref) <= TOL
    explicit = host(B.conv_backward_data(d.with_flags(0), dYg, Wg))
    assert rel_err(got, explicit) <= 1e-2
    assert np.all(got[ref == 0] == 0)              # pixels no window reaches are exactly zero
    assert np.array_equal(got, host(B.conv_backward_data(d, dYg, Wg)))   # deterministic


def test_strided_declines(B):
    # padding, more than 96 filters, a reduction beyond 400: the explicit path runs
    for N, C, H, W, F, k, p in [(2, 3, 35, 35, 8, 11, 2), (2, 3, 35, 35, 97, 11, 0), (2, 40, 15, 15, 8, 3, 0)]:
        d = B.conv_desc(N, C, H, W, F, k, k, (4, 4), (p, p), BF16, B.FLAG_FUSED)
        assert not B.conv_fused_supported(d, B.PASS_FORWARD)
        s = oracle.shape(N, C, H, W, F, k, k, (4, 4), (p, p))
        rng = np.random.default_rng(4)
        X = wl.to_bf16_values(rng.standard_normal((N, C, H, W)))
        Wt = wl.to_bf16_values(0.05 * rng.standard_normal((F, C, k, k)))
        got = host(B.conv_forward(d, gpu(X), gpu(Wt), None))
        assert rel_err(got, oracle.conv_forward(s, X, Wt, None)) <= TOL


def test_fused_stack_matches_explicit_stack(B):
    """The chained CIFAR-shaped stack in bf16: fused and explicit runs agree on outputs and gradients."""
    from paper_1606_04487_amd.stack import ConvStack
    layers = wl.cifar_stack(16)
    t = wl.stack_tensors(layers, seed=5, bf16=True, pooled_out=(4, 4))
    Ws, bs, X, dOut = t["W"], t["bias"], t["X"], t["dY"]
    res = []
    for fused in (False, True):
        st = ConvStack(layers, dtype=B.BF16, ceil_mode=True, skip_first_dgrad=False, fused=fused)
        st.set_parameters(Ws, bs)
        out = st.forward(gpu(X))
        dx = st.backward(gpu(dOut))
        res.append((host(out), host(dx), [host(w) for w in st.dW], st.fwd_fused))
    assert res[1][3][1] and res[1][3][2] and not res[1][3][0]   # conv2, conv3 fused; conv1 (C = 3) not
    assert rel_err(res[1][0], res[0][0]) <= 2e-2
    assert rel_err(res[1][1], res[0][1]) <= 3e-2
    for a, b in zip(res[1][2], res[0][2]):
        assert rel_err(a, b) <= 3e-2


def test_second_stream_model_gradient_is_identical(B):
    """ConvStack(overlap_wgrad=True) runs each layer's model gradient on a second stream beside the data
    gradient; the same kernels on the same inputs: every result bit-identical, step after step."""
    from paper_1606_04487_amd.stack import ConvStack
    layers = wl.cifar_stack(16)
    t = wl.stack_tensors(layers, seed=7, bf16=True, pooled_out=(4, 4))
    res = []
    for overlap in (False, True):
        st = ConvStack(layers, dtype=B.BF16, ceil_mode=True, skip_first_dgrad=False, overlap_wgrad=overlap)
        st.set_parameters(t["W"], t["bias"])
        outs = []
        for _ in range(3):
            out = st.step(gpu(t["X"]), gpu(t["dY"]), 0.01, 0.9)
            outs.append(out.clone())
        torch.cuda.synchronize()
        res.append((outs, [w.clone() for w in st.W], [d.clone() for d in st.dW], st.dXl[0].clone()))
    for a, b in zip(res[0][0], res[1][0]):
        assert torch.equal(a, b)
    for k in (1, 2):
        for a, b in zip(res[0][k], res[1][k]):
            assert torch.equal(a, b)
    assert torch.equal(res[0][3], res[1][3])


@pytest.mark.parametrize("which", ["cifar", "caffenet"])
def test_step_replayed_as_a_hip_graph_is_identical(B, which):
    """A step allocates nothing, clears no memory and waits for nothing, so it can be captured once and replayed
    as a HIP graph (what `bench.py --graph` times).  Every replay, with eager launches and synchronisations of the
    program's own between the replays, must leave exactly what the same number of eager steps leaves."""
    from paper_1606_04487_amd.stack import ConvStack
    if which == "cifar":
        layers, ceil, pooled = wl.cifar_stack(16), True, (4, 4)
    else:
        layers, ceil, pooled = wl.caffenet_stack(8), False, (6, 6)
    t = wl.stack_tensors(layers, seed=9, bf16=True, pooled_out=pooled)
    X = gpu(t["X"])
    dOut = (gpu(t["dY"]).float() * wl.step_upstream_scale(layers[0].N)).to(torch.bfloat16)
    eager = ConvStack(layers, dtype=B.BF16, ceil_mode=ceil, skip_first_dgrad=False)
    replayed = ConvStack(layers, dtype=B.BF16, ceil_mode=ceil, skip_first_dgrad=False)
    for st in (eager, replayed):
        st.set_parameters(t["W"], t["bias"])
        st.step(X, dOut, 0.01, 0.9)          # step 1 eager on both (also warms the capture up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        replayed.step(X, dOut, 0.01, 0.9)    # recorded, not run
    torch.cuda.synchronize()
    for it in range(4):
        eager.step(X, dOut, 0.01, 0.9)       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("W", "b", "VW", "dW", "db", "Y", "dYc"):
            for a, b in zip(getattr(eager, name), getattr(replayed, name)):
                assert torch.equal(a, b), (which, it, name)
        assert torch.equal(eager.dXl[0], replayed.dXl[0]), (which, it)
