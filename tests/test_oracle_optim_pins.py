"""Pins for the oracle's optimizer variants: Nesterov momentum and the
step-size schedules of the paper's experiments.  CPU only."""
import numpy as np
import pytest

from conftest import read_golden
from oracle import gpga_oracle as orc

RNG = np.random.default_rng(2024)


# ---------------------------------------------------------------- Nesterov momentum

def test_nesterov_two_steps_by_hand():
    # n = 1 (no mixing), scalar parameter, prescribed gradients 1 and 2, gamma = 0.1, mu = 0.5:
    # m1 = 1          x1 = 0    - 0.1 (1 + 0.5*1)    = -0.15
    # m2 = 0.5*1 + 2  x2 = -0.15 - 0.1 (2 + 0.5*2.5) = -0.475
    sim = orc.GossipPGA(1, 1, topology="ring", H=0, lr=0.1, momentum=0.5, nesterov=True, storage="f64")
    sim.step(np.array([[1.0]]))
    assert sim.X[0, 0] == pytest.approx(-0.15, abs=1e-16)
    sim.step(np.array([[2.0]]))
    assert sim.X[0, 0] == pytest.approx(-0.475, abs=1e-16)
    assert sim.M[0, 0] == pytest.approx(2.5, abs=1e-16)


@pytest.mark.parametrize("mu", [0.3, 0.9])
def test_nesterov_is_the_look_ahead_recursion_after_a_change_of_variables(mu):
    # Nesterov's accelerated gradient in the look-ahead form
    #     v <- mu v - gamma grad f(theta + mu v) ;  theta <- theta + v
    # written for the look-ahead point x = theta + mu v is the update the oracle implements.
    # Independent loop on a quadratic f(x) = 1/2 x^T Q x - c^T x, one node.
    d, lr = 4, 0.05
    Q = RNG.standard_normal((d, d))
    Q = Q @ Q.T / d + np.eye(d)
    c = RNG.standard_normal(d)
    grad = lambda x: Q @ x - c
    sim = orc.GossipPGA(1, d, topology="none", H=0, lr=lr, momentum=mu, nesterov=True, storage="f64")
    theta, v = np.zeros(d), np.zeros(d)
    for _ in range(40):
        sim.step(grad(sim.X[0])[None, :])
        v = mu * v - lr * grad(theta + mu * v)
        theta = theta + v
        np.testing.assert_allclose(sim.X[0], theta + mu * v, atol=1e-13)
    # and it converges to the minimiser Q^-1 c
    for _ in range(3000):
        sim.step(grad(sim.X[0])[None, :])
    np.testing.assert_allclose(sim.X[0], np.linalg.solve(Q, c), atol=1e-10)


def test_nesterov_with_zero_momentum_is_algorithm_1():
    n, d = 5, 3
    a = orc.GossipPGA(n, d, topology="ring", H=3, lr=0.1, momentum=0.0, nesterov=True, storage="f64")
    b = orc.GossipPGA(n, d, topology="ring", H=3, lr=0.1, momentum=0.0, storage="f64")
    for _ in range(7):
        G = RNG.standard_normal((n, d))
        a.step(G), b.step(G)
        np.testing.assert_array_equal(a.X, b.X)


def test_nesterov_differs_from_heavy_ball_by_gamma_times_g_minus_mu_m():
    # x_nes - x_hb = -gamma (g + mu m' - m') with m' the new buffer, before mixing (W = I)
    n, d, lr, mu = 3, 4, 0.2, 0.8
    X, M, G = (RNG.standard_normal((n, d)) for _ in range(3))
    Yn, Mn = orc.local_update(X, M, G, lr, mu, nesterov=True)
    Yh, Mh = orc.local_update(X, M, G, lr, mu)
    np.testing.assert_array_equal(Mn, Mh)                     # the buffer itself is the same
    np.testing.assert_allclose(Yn - Yh, -lr * (G + (mu - 1.0) * Mh), atol=1e-15)


def test_nesterov_keeps_the_momentum_buffer_local_and_the_mean_recursion():
    # averaging X does not touch M; the node mean follows xbar+ = xbar - gamma mean(g + mu m')
    n, d, lr, mu = 6, 3, 0.1, 0.9
    sim = orc.GossipPGA(n, d, topology="expo1", H=4, lr=lr, momentum=mu, nesterov=True, storage="f64")
    for k in range(9):
        G = RNG.standard_normal((n, d))
        xbar, M_old = sim.X.mean(axis=0), sim.M.copy()
        sim.step(G)
        M_new = mu * M_old + G
        np.testing.assert_allclose(sim.M, M_new, atol=1e-15)
        np.testing.assert_allclose(sim.X.mean(axis=0), xbar - lr * (G + mu * M_new).mean(axis=0), atol=1e-14)
        if (k + 1) % 4 == 0:
            assert (sim.X == sim.X[0]).all()              # all rows identical after the average


# ---------------------------------------------------------------- step-size schedules

def test_step_decay_reproduces_the_halving_rule_of_the_logistic_experiment():
    # Sec. 5.1: gamma starts at 0.2 and is halved every 1000 iterations
    for k_s, lr_s in read_golden("lr_halving.txt"):
        assert orc.lr_step_decay(int(k_s), 0.2, 1000, 0.5) == pytest.approx(float(lr_s), rel=1e-15)


def test_warmup_then_division_by_ten_at_epochs_30_60_90():
    # Sec. 5.2 / App. F.1: warm-up over 5 epochs, divided by 10 at epochs 30, 60, 90 of 120.
    # ImageNet-1k has 1,281,167 training images (Sec. 5.2); total batch 8192 (App. F.1).
    ipe = 1281167 // 8192                      # 156 iterations per epoch
    base, start = 3.2, 0.1
    ms = [30 * ipe, 60 * ipe, 90 * ipe]
    f = lambda k: orc.lr_warmup_milestones(k, base, 5 * ipe, start, ms, 0.1)
    assert f(0) == start
    assert f(5 * ipe) == base
    # constant increments during warm-up
    inc = np.diff([f(k) for k in range(5 * ipe + 1)])
    np.testing.assert_allclose(inc, (base - start) / (5 * ipe), rtol=1e-9)
    assert f(30 * ipe - 1) == base
    assert f(30 * ipe) == pytest.approx(base / 10, rel=1e-15)
    assert f(60 * ipe - 1) == pytest.approx(base / 10, rel=1e-15)
    assert f(60 * ipe) == pytest.approx(base / 100, rel=1e-15)
    assert f(90 * ipe) == pytest.approx(base / 1000, rel=1e-15)
    assert f(120 * ipe - 1) == pytest.approx(base / 1000, rel=1e-15)


def test_polynomial_decay_with_warmup():
    # App. F.1 (BERT phase 1): initial rate 3.75e-4, 112,608 steps, polynomial decay with warm-up
    base, T, Kw = 3.75e-4, 112608, 2000
    f = lambda k, p: orc.lr_poly(k, base, Kw, T, p)
    assert f(0, 0.5) == 0.0 and f(Kw, 0.5) == base and f(T, 0.5) == 0.0 and f(T + 5, 1.0) == 0.0
    assert f(Kw // 2, 1.0) == pytest.approx(base / 2, rel=1e-15)
    mid = Kw + (T - Kw) // 2
    assert f(mid, 1.0) == pytest.approx(base * 0.5, rel=1e-12)           # power 1: a straight line
    assert f(mid, 0.5) == pytest.approx(base * np.sqrt(0.5), rel=1e-12)  # power 1/2: square root of it
    ks = np.arange(Kw, T, 997)
    vals = np.array([f(int(k), 2.0) for k in ks])
    assert (np.diff(vals) < 0).all()                                     # monotone after warm-up


def test_schedule_drives_the_iteration_and_is_stored_as_float32():
    n, d = 4, 3
    sched = lambda k: orc.lr_step_decay(k, 0.2, 3, 0.5)
    sim = orc.GossipPGA(n, d, topology="ring", H=0, lr=sched, momentum=0.0, storage="f32")
    W = orc.mixing_matrix("ring", n)
    X = np.zeros((n, d))
    for k in range(8):
        G = RNG.standard_normal((n, d)).astype(np.float32).astype(np.float64)
        sim.step(G)
        lr32 = float(np.float32(0.2 * 0.5 ** (k // 3)))
        assert sim.lr_at(k) == lr32
        X = (W @ (X - lr32 * G)).astype(np.float32).astype(np.float64)
        np.testing.assert_array_equal(sim.X, X)
