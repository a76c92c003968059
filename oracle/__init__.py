"""CPU oracle for the batched-lowering convolution path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, double-precision implementation of what the GPU library computes, written
from the paper (Omnivore, arXiv 1606.04487: Sec. II-B for BW and the update equations,
Sec. III-A Eq. (conv_full) and App. C for the layer and for lowering).  Only tests, the
smoke check and the bench's CPU-baseline leg may import it; the GPU package never does, and
nothing here imports the GPU package.

`conv_oracle.c` holds the arithmetic (seven-loop convolution and its two adjoints, the
lowering index map, col2im, ReLU, max-pool, the momentum update); this module compiles it
with gcc and wraps it with ctypes.  `lowering_route.py` is a second, independent route
(index-map lowering + matrix product) that the pins use to cross-check the direct loops.

Every function takes float32 (or float-valued) numpy arrays, uses their values exactly,
accumulates in float64 and returns float64 -- except `lower`, which is a copy and returns
the input's dtype, and argmax outputs, which are int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "conv_oracle.c"
_LIB = _HERE / "liboracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile conv_oracle.c into liboracle.so (gcc, OpenMP)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Shape(ctypes.Structure):
    """Mirror of `oc_shape`: N, C, H, W, F, kh, kw, sh, sw, ph, pw."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "F", "kh", "kw", "sh", "sw", "ph", "pw")]


def shape(N, C, H, W, F, kh, kw=None, stride=1, pad=0) -> Shape:
    kw = kh if kw is None else kw
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    return Shape(N, C, H, W, F, kh, kw, sh, sw, ph, pw)


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(str(_LIB))
        _lib.oc_out_dims.restype = ctypes.c_int
        _lib.oc_pool_out_dim.restype = ctypes.c_int
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oc_num_threads())


def out_dims(s: Shape):
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    if _load().oc_out_dims(ctypes.byref(s), ctypes.byref(ho), ctypes.byref(wo)) != 0:
        raise ValueError("invalid convolution shape")
    return ho.value, wo.value


def conv_forward(s: Shape, X, Wt, bias=None):
    """Y[n,f,oy,ox] = bias[f] + sum_{c,ky,kx} X[n,c,oy*s-p+ky,ox*s-p+kx] W[f,c,ky,kx]
    (Sec. III-A Eq. (conv_full); zero outside the input)."""
    ho, wo = out_dims(s)
    X, xp = _f32(X)
    Wt, wp = _f32(Wt)
    bp = None
    if bias is not None:
        bias, bp = _f32(bias)
    Y = np.empty((s.N, s.F, ho, wo), dtype=np.float64)
    _load().oc_conv_forward(ctypes.byref(s), xp, wp, bp, _ptr(Y))
    return Y


def conv_backward_data(s: Shape, dY, Wt):
    """Gradient w.r.t. the layer input (Sec. II-B, the BW operation)."""
    dY, gp = _f32(dY)
    Wt, wp = _f32(Wt)
    dX = np.empty((s.N, s.C, s.H, s.W), dtype=np.float64)
    _load().oc_conv_backward_data(ctypes.byref(s), gp, wp, _ptr(dX))
    return dX


def conv_backward_weights(s: Shape, X, dY):
    """Gradient w.r.t. the model, summed over the batch (Sec. II-B)."""
    X, xp = _f32(X)
    dY, gp = _f32(dY)
    dW = np.empty((s.F, s.C, s.kh, s.kw), dtype=np.float64)
    _load().oc_conv_backward_weights(ctypes.byref(s), xp, gp, _ptr(dW))
    return dW


def bias_grad(s: Shape, dY):
    dY, gp = _f32(dY)
    db = np.empty((s.F,), dtype=np.float64)
    _load().oc_bias_grad(ctypes.byref(s), gp, _ptr(db))
    return db


def _idx(idx):
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    return idx, idx.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(idx.size)


def conv_forward_at(s: Shape, X, Wt, bias, flat_idx):
    """Entries of Y at the given flat indices (row-major [N][F][Ho][Wo])."""
    X, xp = _f32(X)
    Wt, wp = _f32(Wt)
    bp = None
    if bias is not None:
        bias, bp = _f32(bias)
    idx, ip, cnt = _idx(flat_idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_forward_at(ctypes.byref(s), xp, wp, bp, ip, cnt, _ptr(out))
    return out


def conv_backward_data_at(s: Shape, dY, Wt, flat_idx):
    """Entries of dX at the given flat indices (row-major [N][C][H][W])."""
    dY, gp = _f32(dY)
    Wt, wp = _f32(Wt)
    idx, ip, cnt = _idx(flat_idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_backward_data_at(ctypes.byref(s), gp, wp, ip, cnt, _ptr(out))
    return out


def conv_backward_weights_at(s: Shape, X, dY, flat_idx):
    """Entries of dW at the given flat indices (row-major [F][C][kh][kw])."""
    X, xp = _f32(X)
    dY, gp = _f32(dY)
    idx, ip, cnt = _idx(flat_idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_backward_weights_at(ctypes.byref(s), xp, gp, ip, cnt, _ptr(out))
    return out


def lower(s: Shape, X):
    """D-hat, row-major [C*kh*kw][N*Ho*Wo] (App. C, lowering phase); a copy of X's values."""
    ho, wo = out_dims(s)
    X, xp = _f32(X)
    D = np.empty((s.C * s.kh * s.kw, s.N * ho * wo), dtype=np.float32)
    _load().oc_lower(ctypes.byref(s), xp, _ptr(D))
    return D


def col2im(s: Shape, dDhat):
    """Transpose of the lowering map: sums every D-hat-shaped entry into its source pixel."""
    dDhat, dp = _f32(dDhat)
    dX = np.empty((s.N, s.C, s.H, s.W), dtype=np.float64)
    _load().oc_col2im(ctypes.byref(s), dp, _ptr(dX))
    return dX


def matmul(A, B):
    """Triple-loop float64 matrix product."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.empty((m, n), dtype=np.float64)
    _load().oc_matmul(ctypes.c_int64(m), ctypes.c_int64(k), ctypes.c_int64(n),
                      _ptr(A), _ptr(B), _ptr(C))
    return C


def relu_forward(x):
    x, xp = _f32(x)
    y = np.empty(x.shape, dtype=np.float64)
    _load().oc_relu_forward(ctypes.c_int64(x.size), xp, _ptr(y))
    return y


def relu_backward(x, dy):
    """dx = dy where the ReLU *input* (equivalently its output) is > 0, else 0."""
    x, xp = _f32(x)
    dy, gp = _f32(dy)
    dx = np.empty(x.shape, dtype=np.float64)
    _load().oc_relu_backward(ctypes.c_int64(x.size), xp, gp, _ptr(dx))
    return dx


def pool_out_dim(n, k, stride, ceil_mode):
    o = _load().oc_pool_out_dim(int(n), int(k), int(stride), int(bool(ceil_mode)))
    if o < 0:
        raise ValueError("invalid pooling shape")
    return o


def maxpool_forward(x, k=3, stride=2, ceil_mode=True):
    """Max-pool the last two axes; returns (y float64, argmax int32 flat iy*W+ix)."""
    x, xp = _f32(x)
    H, W = x.shape[-2:]
    planes = int(np.prod(x.shape[:-2], dtype=np.int64))
    ho, wo = pool_out_dim(H, k, stride, ceil_mode), pool_out_dim(W, k, stride, ceil_mode)
    y = np.empty(x.shape[:-2] + (ho, wo), dtype=np.float64)
    am = np.empty(x.shape[:-2] + (ho, wo), dtype=np.int32)
    _load().oc_maxpool_forward(ctypes.c_int64(planes), H, W, k, stride, int(bool(ceil_mode)),
                               xp, _ptr(y), _ptr(am))
    return y, am


def maxpool_backward(dy, argmax, H, W):
    dy, gp = _f32(dy)
    argmax = np.ascontiguousarray(argmax, dtype=np.int32)
    ho, wo = dy.shape[-2:]
    planes = int(np.prod(dy.shape[:-2], dtype=np.int64))
    dx = np.empty(dy.shape[:-2] + (H, W), dtype=np.float64)
    _load().oc_maxpool_backward(ctypes.c_int64(planes), H, W, ho, wo, gp, _ptr(argmax), _ptr(dx))
    return dx


def sgd_momentum(W0, V0, G, lr, mu, weight_decay=0.0):
    """V1 = mu*V0 - lr*(G + lambda*W0); W1 = W0 + V1 (Sec. II-B Eq. (update2), (update1))."""
    W0, wp = _f32(W0)
    V0, vp = _f32(V0)
    G, gp = _f32(G)
    W1 = np.empty(W0.shape, dtype=np.float64)
    V1 = np.empty(W0.shape, dtype=np.float64)
    _load().oc_sgd_momentum(ctypes.c_int64(W0.size), wp, vp, gp, ctypes.c_double(lr),
                            ctypes.c_double(mu), ctypes.c_double(weight_decay),
                            _ptr(W1), _ptr(V1))
    return W1, V1


def conv_flops(N, C, H, W, F, kh, kw=None, stride=1, pad=0):
    """Multiply-add count x2 of the layer's matrix product: 2 * (N*Ho*Wo) * (C*kh*kw) * F."""
    s = shape(N, C, H, W, F, kh, kw, stride, pad)
    ho, wo = out_dims(s)
    return 2 * (s.N * ho * wo) * (s.C * s.kh * s.kw) * s.F


def lrn_forward(x, size=5, alpha=1e-4, beta=0.75, k=1.0):
    """Local response normalisation across channels of x [N][C][...]:
    y = x * (k + alpha/size * sum over the channel window of x^2)^(-beta)."""
    if size % 2 != 1:
        raise ValueError("the channel window must have an odd size")
    x, xp = _f32(x)
    N, C = x.shape[:2]
    plane = int(np.prod(x.shape[2:], dtype=np.int64))
    y = np.empty(x.shape, dtype=np.float64)
    _load().oc_lrn_forward(ctypes.c_int64(N), ctypes.c_int64(C), ctypes.c_int64(plane), ctypes.c_int32(size),
                           ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_double(k), xp, _ptr(y))
    return y


def lrn_backward(x, dy, size=5, alpha=1e-4, beta=0.75, k=1.0):
    """Gradient of lrn_forward w.r.t. x given the gradient dy w.r.t. its output."""
    if size % 2 != 1:
        raise ValueError("the channel window must have an odd size")
    x, xp = _f32(x)
    dy, gp = _f32(dy)
    N, C = x.shape[:2]
    plane = int(np.prod(x.shape[2:], dtype=np.int64))
    dx = np.empty(x.shape, dtype=np.float64)
    _load().oc_lrn_backward(ctypes.c_int64(N), ctypes.c_int64(C), ctypes.c_int64(plane), ctypes.c_int32(size),
                            ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_double(k), xp, gp, _ptr(dx))
    return dx


def philox4x64(counter, key):
    """One block of Philox4x64-10: four 64-bit words from a 4-word counter and a 2-word key."""
    c = (ctypes.c_uint64 * 4)(*[int(v) for v in counter])
    k = (ctypes.c_uint64 * 2)(*[int(v) for v in key])
    out = (ctypes.c_uint64 * 4)()
    _load().oc_philox4x64(c, k, out)
    return [int(v) for v in out]


def dropout_threshold(p):
    lib = _load()
    lib.oc_dropout_threshold.restype = ctypes.c_uint32
    return int(lib.oc_dropout_threshold(ctypes.c_double(p)))


def dropout_mask(count, p, seed, stream=0):
    """uint8 keep-mask of `count` elements (1 = kept) for drop probability p."""
    keep = np.empty(int(count), dtype=np.uint8)
    _load().oc_dropout_mask(ctypes.c_int64(count), ctypes.c_double(p), ctypes.c_uint64(seed), ctypes.c_uint64(stream),
                            _ptr(keep))
    return keep


def dropout_apply(x, p, seed, stream=0):
    """keep ? x / (1 - p) : 0 elementwise over the flattened x; serves forward (x) and backward (dy)."""
    x, xp = _f32(x)
    y = np.empty(x.shape, dtype=np.float64)
    _load().oc_dropout_apply(ctypes.c_int64(x.size), ctypes.c_double(p), ctypes.c_uint64(seed), ctypes.c_uint64(stream),
                             xp, _ptr(y))
    return y
