"""Second CPU route: lowering + one matrix product + lifting -- TEST INFRASTRUCTURE ONLY.

App. C ("Convolution by Lowering and GEMM") describes the layer as three phases: build the
replicated matrix D-hat (and the reshaped model K-hat), multiply, and map the product back
to a tensor.  This module does exactly that with pure-Python index loops and numpy's
float64 matmul, for tiny inputs.  It exists so that the direct seven-loop oracle in
conv_oracle.c can be checked against an independently written formulation; it shares no
code with it (nor with the GPU library).
"""
from __future__ import annotations

import numpy as np


def out_dims(H, W, kh, kw, sh, sw, ph, pw):
    return (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1


def lower(X, kh, kw, sh, sw, ph, pw):
    """D-hat [C*kh*kw][N*Ho*Wo] by the index map, one Python assignment per entry."""
    N, C, H, W = X.shape
    Ho, Wo = out_dims(H, W, kh, kw, sh, sw, ph, pw)
    D = np.zeros((C * kh * kw, N * Ho * Wo), dtype=X.dtype)
    for c in range(C):
        for ky in range(kh):
            for kx in range(kw):
                r = (c * kh + ky) * kw + kx
                for n in range(N):
                    for oy in range(Ho):
                        iy = oy * sh - ph + ky
                        if not 0 <= iy < H:
                            continue
                        for ox in range(Wo):
                            ix = ox * sw - pw + kx
                            if 0 <= ix < W:
                                D[r, (n * Ho + oy) * Wo + ox] = X[n, c, iy, ix]
    return D


def col2im(dD, N, C, H, W, kh, kw, sh, sw, ph, pw):
    """Adds every entry of a D-hat-shaped matrix back onto the pixel it was copied from."""
    Ho, Wo = out_dims(H, W, kh, kw, sh, sw, ph, pw)
    dX = np.zeros((N, C, H, W), dtype=np.float64)
    for c in range(C):
        for ky in range(kh):
            for kx in range(kw):
                r = (c * kh + ky) * kw + kx
                for n in range(N):
                    for oy in range(Ho):
                        iy = oy * sh - ph + ky
                        if not 0 <= iy < H:
                            continue
                        for ox in range(Wo):
                            ix = ox * sw - pw + kx
                            if 0 <= ix < W:
                                dX[n, c, iy, ix] += dD[r, (n * Ho + oy) * Wo + ox]
    return dX


def lift(Rhat, N, F, Ho, Wo):
    """R-hat [F][N*Ho*Wo] -> R [N][F][Ho][Wo] (a pure re-indexing)."""
    return np.ascontiguousarray(Rhat.reshape(F, N, Ho, Wo).transpose(1, 0, 2, 3))


def unlift(R):
    """R [N][F][Ho][Wo] -> R-hat [F][N*Ho*Wo]."""
    N, F, Ho, Wo = R.shape
    return np.ascontiguousarray(R.transpose(1, 0, 2, 3).reshape(F, N * Ho * Wo))


def conv_forward(X, Wt, bias, sh, sw, ph, pw):
    N, C, H, W = X.shape
    F, _, kh, kw = Wt.shape
    Ho, Wo = out_dims(H, W, kh, kw, sh, sw, ph, pw)
    D = lower(X.astype(np.float64), kh, kw, sh, sw, ph, pw)
    K = Wt.astype(np.float64).reshape(F, C * kh * kw)
    R = K @ D
    if bias is not None:
        R = R + np.asarray(bias, dtype=np.float64)[:, None]
    return lift(R, N, F, Ho, Wo)


def conv_backward_data(dY, Wt, H, W, sh, sw, ph, pw):
    N = dY.shape[0]
    F, C, kh, kw = Wt.shape
    K = Wt.astype(np.float64).reshape(F, C * kh * kw)
    dD = K.T @ unlift(dY.astype(np.float64))
    return col2im(dD, N, C, H, W, kh, kw, sh, sw, ph, pw)


def conv_backward_weights(X, dY, kh, kw, sh, sw, ph, pw):
    N, C, H, W = X.shape
    F = dY.shape[1]
    D = lower(X.astype(np.float64), kh, kw, sh, sw, ph, pw)
    return (unlift(dY.astype(np.float64)) @ D.T).reshape(F, C, kh, kw)
