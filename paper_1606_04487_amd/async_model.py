"""Models of the paper's trade-off space, on the CPU (they are models, not part of the GPU path).

* `hardware_efficiency(g, t_conv, t_fc)`: the iteration-time model HE(g) of Sec. IV-B -- with g compute groups
  the FC server is either saturated (time per iteration t_fc) or waits for the groups
  ((t_conv(k) + t_fc) / g).
* `simulate_async_sgd(...)`: g asynchronous groups with exponentially distributed step times (assumption A2 of
  Sec. IV-C) running plain SGD (explicit momentum 0) on a shared model.  Each group reads the model, takes an
  exponentially distributed time to compute the gradient AT THE MODEL IT READ, applies
  V = -eta * gradient, W += V (Eq. (update2), (update1) with mu = 0) and reads again.  Theorem 1 says the
  expected update then carries an implicit momentum of 1 - 1/g:
      E V(t+1) = (1 - 1/g) E V(t) - (eta / g) E grad(W(t)),
  which `implicit_momentum_reference` iterates for a quadratic loss (whose gradient is linear, so the
  expectation passes through it).
"""
from __future__ import annotations

from typing import Callable, Tuple

import numpy as np


def hardware_efficiency(g: int, t_conv: Callable[[int], float], t_fc: float, n_devices: int) -> Tuple[float, str]:
    """HE(g) = max(t_fc, (t_conv(k) + t_fc) / g) with k = n_devices / g devices per group (Sec. IV-B).
    Returns the predicted time per iteration and which phase is saturated."""
    if g < 1 or n_devices % g != 0:
        raise ValueError("g must divide the number of conv devices")
    k = n_devices // g
    conv_bound = (t_conv(k) + t_fc) / g
    return (t_fc, "fc") if t_fc >= conv_bound else (conv_bound, "conv")


def simulate_async_sgd(A: np.ndarray, w_star: np.ndarray, w0: np.ndarray, eta: float, g: int, steps: int,
                       runs: int, seed: int = 1):
    """Monte-Carlo simulation of g asynchronous groups on the loss 0.5 (W - w*)^T A (W - w*).

    Returns (W, staleness): W[t] is the model after t updates averaged over `runs` independent runs
    (shape [steps + 1, d]); staleness[r, t] is the number of updates applied by others between the read
    and the write of the group that made update t in run r."""
    rng = np.random.default_rng(seed)
    d = w0.shape[0]
    W = np.tile(w0, (runs, 1)).astype(np.float64)                 # current model of each run
    read = np.tile(w0, (runs, g, 1)).astype(np.float64)           # the model each group last read
    read_at = np.zeros((runs, g), dtype=np.int64)                 # ... and the update count at that moment
    finish = rng.exponential(1.0, size=(runs, g))                 # when each group's current step ends
    mean_W = np.empty((steps + 1, d))
    mean_W[0] = w0
    staleness = np.empty((runs, steps), dtype=np.int64)
    rows = np.arange(runs)
    for t in range(steps):
        who = np.argmin(finish, axis=1)                           # the group that finishes first, per run
        stale = read[rows, who]
        grad = (stale - w_star) @ A.T                             # gradient at the stale model
        W = W - eta * grad                                        # V = -eta * grad (mu = 0); W += V
        staleness[:, t] = t - read_at[rows, who]
        read[rows, who] = W                                       # read the fresh model, start the next step
        read_at[rows, who] = t + 1
        finish[rows, who] += rng.exponential(1.0, size=runs)
        mean_W[t + 1] = W.mean(axis=0)
    return mean_W, staleness


def implicit_momentum_reference(A: np.ndarray, w_star: np.ndarray, w0: np.ndarray, eta: float, g: int, steps: int):
    """Theorem 1 iterated for a quadratic loss: momentum SGD with momentum 1 - 1/g and step eta / g."""
    w = w0.astype(np.float64).copy()
    v = np.zeros_like(w)
    out = [w.copy()]
    for _ in range(steps):
        v = (1.0 - 1.0 / g) * v - (eta / g) * (A @ (w - w_star))
        w = w + v
        out.append(w.copy())
    return np.array(out)
