"""CPU tests of the trade-off models (Sec. IV-B hardware efficiency, Sec. IV-C implicit momentum)."""
import numpy as np

import oracle
from paper_1606_04487_amd import async_model as am

A = np.array([[1.0, 0.2], [0.2, 0.5]])
W_STAR = np.array([1.0, -2.0])
W0 = np.array([4.0, 3.0])


def test_hardware_efficiency_model_cases():
    t_conv = lambda k: 8.0 / k + 0.5          # a group of k devices: perfect split plus a fixed cost
    # one group of 8: the conv phase is the bottleneck, time = (t_conv(8) + t_fc) / 1
    t, mode = am.hardware_efficiency(1, t_conv, 1.0, 8)
    assert mode == "conv" and abs(t - (1.5 + 1.0)) < 1e-12
    # eight groups of 1: (8.5 + 1) / 8 = 1.1875 > t_fc = 1
    t, mode = am.hardware_efficiency(8, t_conv, 1.0, 8)
    assert mode == "conv" and abs(t - 9.5 / 8) < 1e-12
    # a slow FC server saturates: time per iteration is t_fc whatever the groups do
    t, mode = am.hardware_efficiency(8, t_conv, 2.0, 8)
    assert mode == "fc" and t == 2.0
    # HE(g) never drops below t_fc and is non-increasing in g here
    times = [am.hardware_efficiency(g, t_conv, 1.0, 8)[0] for g in (1, 2, 4, 8)]
    assert all(a >= b for a, b in zip(times, times[1:])) and min(times) >= 1.0


def test_one_group_is_plain_sgd_exactly():
    mean_W, stale = am.simulate_async_sgd(A, W_STAR, W0, 0.3, 1, 30, 7)
    w = W0.copy()
    for t in range(30):
        w = w - 0.3 * (A @ (w - W_STAR))
        assert np.allclose(mean_W[t + 1], w, rtol=0, atol=1e-12)
    assert not stale.any()
    assert np.allclose(am.implicit_momentum_reference(A, W_STAR, W0, 0.3, 1, 30), mean_W, atol=1e-12)


def test_staleness_is_geometric_with_mean_g_minus_one():
    g = 4
    _, stale = am.simulate_async_sgd(A, W_STAR, W0, 0.05, g, 120, 4000, seed=3)
    s = stale[:, 40:].ravel()                 # past the start-up transient
    assert abs(s.mean() - (g - 1)) < 0.05
    for j in range(6):                        # P(staleness = j) = (1/g) (1 - 1/g)^j
        assert abs(np.mean(s == j) - (1 / g) * (1 - 1 / g) ** j) < 0.01


def test_asynchrony_acts_as_momentum_one_minus_one_over_g():
    """Theorem 1, checked as the identity it states: with V(t+1) = W(t+1) - W(t) averaged over many runs,
    E V(t+1) = (1 - 1/g) E V(t) - (eta/g) grad(E W(t)) holds once the start-up transient (all groups begin
    with the same fresh model) has passed -- and the same data are far from plain SGD with step eta/g."""
    eta, steps, runs = 0.4, 80, 40000
    for g in (2, 4, 8):
        mean_W, _ = am.simulate_async_sgd(A, W_STAR, W0, eta, g, steps, runs, seed=11)
        V = np.diff(mean_W, axis=0)                                   # V[t] = E V(t+1)
        t = np.arange(5 * g, steps - 1)
        grad = (mean_W[t + 1] - W_STAR) @ A.T                         # gradient at E W(t+1): the loss is quadratic
        with_momentum = V[t + 1] - ((1 - 1 / g) * V[t] - (eta / g) * grad)
        without = V[t + 1] - (-(eta / g) * grad)
        scale = np.abs(V).max()                                       # Monte-Carlo noise is set by the whole run's step size
        assert np.abs(with_momentum).max() / scale < 0.03, (g, np.abs(with_momentum).max() / scale)
        assert np.abs(without).max() > 10 * np.abs(with_momentum).max(), g
        # the recursion the theorem predicts is momentum SGD (Eq. (update2), (update1)) with mu = 1 - 1/g and
        # step eta/g: iterate it through the oracle's update rule and through the model's own reference
        ref = am.implicit_momentum_reference(A, W_STAR, W0, eta, g, steps)
        w, v = W0.astype(np.float32), np.zeros(2, dtype=np.float32)
        for _ in range(steps):
            gr = (A @ (w.astype(np.float64) - W_STAR)).astype(np.float32)
            w, v = oracle.sgd_momentum(w, v, gr, np.float32(eta / g), np.float32(1 - 1 / g), 0.0)
        assert np.allclose(w, ref[-1], atol=1e-3)
