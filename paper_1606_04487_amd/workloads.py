"""Seeded synthetic workloads shaped like the paper's CNN layers.

This module only describes shapes and draws random tensors; it contains none of the
method's arithmetic and is the one piece shared by the GPU tests, the bench and the CPU
oracle's callers.  Shapes: the CIFAR-style and CaffeNet-style (AlexNet with grouping
removed, App. F "Network" notes) convolution stacks the paper trains, batch 128 and 256
(App. E, batch-size selection).  Values: inputs U[-1,1) or N(0,1), weights and biases
N(0, sigma=0.01) (App. F: Gaussian with standard deviation 0.01), upstream gradients N(0,1).
Draw order per layer is X, W, bias, dY from numpy's PCG64 seeded with `seed`
(default 1, the seed the paper fixes for its runs).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class ConvLayer:
    """One convolution layer: input [N][C][H][W], weights [F][C][k][k], stride s, zero pad p."""
    name: str
    N: int
    C: int
    H: int
    W: int
    F: int
    k: int
    s: int = 1
    p: int = 0
    pool_after: bool = False      # 3x3 stride-2 max-pool follows the ReLU
    relu: bool = True             # ReLU on the layer's output (the last fully connected layer has none)
    lrn_after: bool = False       # normalisation across 5 channels follows the pool (alpha 1e-4, beta 0.75, k 1)
    dropout_after: float = 0.0    # drop probability of a dropout layer that follows (0: none)

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.p - self.k) // self.s + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.p - self.k) // self.s + 1

    @property
    def M(self) -> int:           # columns of D-hat
        return self.N * self.Ho * self.Wo

    @property
    def K(self) -> int:           # rows of D-hat
        return self.C * self.k * self.k

    @property
    def gemm_flops(self) -> int:  # one of the layer's three matrix products
        return 2 * self.M * self.K * self.F

    def with_batch(self, N: int) -> "ConvLayer":
        return replace(self, N=N)


def single_layer_config() -> ConvLayer:
    """Small single layer (fwd+bwd, with bias): N=8, 3x32x32, 32 filters 5x5, pad 2."""
    return ConvLayer("single", 8, 3, 32, 32, 32, 5, 1, 2)


def cifar_stack(N: int = 128) -> List[ConvLayer]:
    """CIFAR-style stack: three 5x5 pad-2 convolutions, each followed by ReLU and a 3x3/2
    max-pool with a border-clipped last window (32 -> 16 -> 8 -> 4)."""
    return [
        ConvLayer("conv1", N, 3, 32, 32, 32, 5, 1, 2, True),
        ConvLayer("conv2", N, 32, 16, 16, 32, 5, 1, 2, True),
        ConvLayer("conv3", N, 32, 8, 8, 64, 5, 1, 2, True),
    ]


def caffenet_stack(N: int = 256) -> List[ConvLayer]:
    """CaffeNet-shaped conv1..conv5 (no grouping); pools after conv1, conv2 and conv5."""
    return [
        ConvLayer("conv1", N, 3, 227, 227, 96, 11, 4, 0, True),
        ConvLayer("conv2", N, 96, 27, 27, 256, 5, 1, 2, True),
        ConvLayer("conv3", N, 256, 13, 13, 384, 3, 1, 1, False),
        ConvLayer("conv4", N, 384, 13, 13, 384, 3, 1, 1, False),
        ConvLayer("conv5", N, 384, 13, 13, 256, 3, 1, 1, True),
    ]


def step_upstream_scale(N: int) -> float:
    """Power of two that the N(0,1) upstream gradient of a REPEATED training step is multiplied with.

    The stack's objective <output, dOut> is linear in the output and multilinear in the layers' weights,
    and the model gradients are summed over the batch (Sec. II-B), so momentum steps with the unscaled
    draw grow the weights without bound: at batch 256 with lr 0.01 and momentum 0.9 every weight is NaN
    after four steps.  Times 2^-18 / N (N rounded up to a power of two) one step moves a weight by about
    1e-7 of its standard deviation, so tens of thousands of steps leave every tensor in the distribution it was
    drawn from.  A power of two changes exponents only: the values keep the mantissas of the seeded draw
    in fp32 and in bf16."""
    import math
    return 2.0 ** -(18 + max(0, math.ceil(math.log2(N))))


def caffenet_full(N: int = 256) -> List[ConvLayer]:
    """The whole CaffeNet-shaped network (Sec. II-C: conv phase, then FC phase): conv1..conv5 as above with the
    two normalisation layers after the first two pools, then FC6 (the convolution whose 6 x 6 window covers the
    whole 256 x 6 x 6 image), FC7 and FC8 (1 x 1 convolutions on 1 x 1 images), dropout 0.5 after FC6 and FC7."""
    conv = caffenet_stack(N)
    conv[0] = replace(conv[0], lrn_after=True)
    conv[1] = replace(conv[1], lrn_after=True)
    return conv + [
        ConvLayer("fc6", N, 256, 6, 6, 4096, 6, 1, 0, dropout_after=0.5),
        ConvLayer("fc7", N, 4096, 1, 1, 4096, 1, 1, 0, dropout_after=0.5),
        ConvLayer("fc8", N, 4096, 1, 1, 1000, 1, 1, 0, relu=False),
    ]


def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bf16 value (ties to even); returned as float32."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(
        torch.float32).numpy()


def layer_tensors(layer: ConvLayer, seed: int = 1, x_dist: str = "normal", bf16: bool = False,
                  with_bias: bool = True, rng: Optional[np.random.Generator] = None
                  ) -> Dict[str, np.ndarray]:
    """X, W, bias, dY for one layer as float32 arrays (bf16-representable if `bf16`)."""
    rng = np.random.default_rng(seed) if rng is None else rng
    if x_dist == "uniform":
        X = rng.uniform(-1.0, 1.0, size=(layer.N, layer.C, layer.H, layer.W)).astype(np.float32)
    else:
        X = rng.standard_normal((layer.N, layer.C, layer.H, layer.W), dtype=np.float32)
    W = (0.01 * rng.standard_normal((layer.F, layer.C, layer.k, layer.k), dtype=np.float32)
         ).astype(np.float32)
    bias = (0.01 * rng.standard_normal((layer.F,), dtype=np.float32)).astype(np.float32)
    dY = rng.standard_normal((layer.N, layer.F, layer.Ho, layer.Wo), dtype=np.float32)
    if bf16:
        X, W, dY = to_bf16_values(X), to_bf16_values(W), to_bf16_values(dY)
    out = {"X": X, "W": W, "dY": dY}
    if with_bias:
        out["bias"] = bias          # biases and weight gradients stay fp32 in both modes
    return out


def stack_tensors(layers: List[ConvLayer], seed: int = 1, x_dist: str = "normal",
                  bf16: bool = False, pooled_out: Optional[tuple] = None) -> Dict[str, object]:
    """Input image batch, per-layer W/bias, and the upstream gradient at the stack's output.

    `pooled_out` is the (H, W) of the last layer's output after its pool (if any); the
    caller computes it with the pooling rule it uses."""
    rng = np.random.default_rng(seed)
    first = layers[0]
    if x_dist == "uniform":
        X = rng.uniform(-1.0, 1.0, size=(first.N, first.C, first.H, first.W)).astype(np.float32)
    else:
        X = rng.standard_normal((first.N, first.C, first.H, first.W), dtype=np.float32)
    Ws, bs = [], []
    for L in layers:
        Ws.append((0.01 * rng.standard_normal((L.F, L.C, L.k, L.k), dtype=np.float32)
                   ).astype(np.float32))
        bs.append((0.01 * rng.standard_normal((L.F,), dtype=np.float32)).astype(np.float32))
    last = layers[-1]
    oh, ow = pooled_out if pooled_out is not None else (last.Ho, last.Wo)
    dY = rng.standard_normal((last.N, last.F, oh, ow), dtype=np.float32)
    if bf16:
        X, dY = to_bf16_values(X), to_bf16_values(dY)
        Ws = [to_bf16_values(w) for w in Ws]
    return {"X": X, "W": Ws, "bias": bs, "dY": dY}
