"""Pins for the oracle's further mixing graphs: grid, static exponential graph and
an arbitrary doubly stochastic W.  CPU only."""
import math

import numpy as np
import pytest

from oracle import gpga_oracle as orc

RNG = np.random.default_rng(777)


@pytest.mark.parametrize("topology", ["grid", "expo"])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 6, 7, 12, 20, 50, 64, 100])
def test_W_is_nonnegative_doubly_stochastic_and_contains_self(topology, n):
    W = orc.mixing_matrix(topology, n)
    assert (W >= 0).all()
    np.testing.assert_allclose(W.sum(axis=1), 1.0, atol=1e-15)
    np.testing.assert_allclose(W.sum(axis=0), 1.0, atol=1e-15)
    assert (np.diag(W) > 0).all()


def test_grid_shape_is_the_most_square_factorisation():
    assert orc.grid_shape(64) == (8, 8)
    assert orc.grid_shape(20) == (4, 5)
    assert orc.grid_shape(50) == (5, 10)
    assert orc.grid_shape(1024) == (32, 32)
    assert orc.grid_shape(13) == (1, 13)
    assert orc.grid_shape(1) == (1, 1)


def test_grid_neighbourhood_is_self_plus_four_with_equal_weights():
    n = 20                                   # 4 x 5
    r, c = orc.grid_shape(n)
    W = orc.mixing_matrix("grid", n)
    for a in range(r):
        for b in range(c):
            i = a * c + b
            want = {i, ((a - 1) % r) * c + b, ((a + 1) % r) * c + b, a * c + (b - 1) % c, a * c + (b + 1) % c}
            nz = set(np.nonzero(W[i])[0])
            assert nz == want and len(nz) == 5          # |N_i| = 5 (Sec. 3.3)
            np.testing.assert_allclose(W[i, sorted(nz)], 0.2)
    np.testing.assert_allclose(W, W.T)                   # undirected graph


def test_grid_degenerate_shapes_fold_coinciding_neighbours():
    # 1 x n: up and down neighbours are the node itself -> 3/5 on the diagonal, ring otherwise
    W = orc.mixing_matrix("grid", 7)
    for i in range(7):
        assert W[i, i] == pytest.approx(0.6) and W[i, (i + 1) % 7] == pytest.approx(0.2)
    # 2 x 2: both vertical neighbours coincide, both horizontal ones too
    W = orc.mixing_matrix("grid", 4)
    np.testing.assert_allclose(W[0], [0.2, 0.4, 0.4, 0.0])


def test_grid_beta_closed_form_and_order_one_over_n():
    for n in (20, 50, 64, 100, 144):
        r, c = orc.grid_shape(n)
        lam = [(1 + 2 * math.cos(2 * math.pi * p / r) + 2 * math.cos(2 * math.pi * q / c)) / 5
               for p in range(r) for q in range(c) if (p, q) != (0, 0)]
        assert orc.beta_of(orc.mixing_matrix("grid", n)) == pytest.approx(max(abs(v) for v in lam), abs=1e-12)
    # 1 - beta = O(1/n) (Sec. 3.3, transient-time tables): square grids, n x 4 -> gap / 4
    g1 = 1 - orc.beta_of(orc.mixing_matrix("grid", 256))
    g2 = 1 - orc.beta_of(orc.mixing_matrix("grid", 1024))
    assert g1 / g2 == pytest.approx(4.0, rel=2e-2)
    assert g2 * 1024 == pytest.approx(4 * math.pi ** 2 / 5, rel=1e-2)


def test_grid_eigenvector_is_scaled_by_its_eigenvalue():
    n, p, q = 20, 1, 2
    r, c = orc.grid_shape(n)
    a, b = np.divmod(np.arange(n), c)
    v = np.cos(2 * np.pi * (p * a / r + q * b / c))[:, None]
    X1, _ = orc.gossip_pga_step(v, np.zeros_like(v), np.zeros_like(v), 0, topology="grid", H=0, lr=0.1)
    lam = (1 + 2 * math.cos(2 * math.pi * p / r) + 2 * math.cos(2 * math.pi * q / c)) / 5
    np.testing.assert_allclose(X1, lam * v, atol=1e-15)


def test_static_exponential_graph_structure_and_beta():
    n = 12
    tau = 4
    W = orc.mixing_matrix("expo", n)
    for i in range(n):
        nz = set(np.nonzero(W[i])[0])
        assert nz == {i} | {(i + (1 << j)) % n for j in range(tau)}
        np.testing.assert_allclose(W[i, sorted(nz)], 1.0 / (tau + 1))
    # circulant => normal: beta = max modulus of the non-principal eigenvalues
    for n in (12, 20, 50, 100):
        tau = orc.one_peer_tau(n)
        w = np.exp(2j * np.pi * np.arange(1, n) / n)
        lam = (1 + sum(w ** (1 << j) for j in range(tau))) / (tau + 1)
        assert orc.beta_of(orc.mixing_matrix("expo", n)) == pytest.approx(np.abs(lam).max(), abs=1e-12)
    # n a power of two: beta = (tau - 1) / (tau + 1)
    for tau in (2, 3, 6, 8):
        assert orc.beta_of(orc.mixing_matrix("expo", 1 << tau)) == pytest.approx((tau - 1) / (tau + 1), abs=1e-12)


@pytest.mark.parametrize("n", [20, 50, 100])
def test_connectivity_order_exponential_then_grid_then_ring(n):
    # App. F.2: the exponential graph has the smallest beta, the ring the largest
    b = {t: orc.beta_of(orc.mixing_matrix(t, n)) for t in ("expo", "grid", "ring")}
    assert b["expo"] < b["grid"] < b["ring"] < 1.0


def _birkhoff(n, terms=4):
    """A random doubly stochastic matrix: convex combination of permutation matrices."""
    w = RNG.random(terms + 1)
    w /= w.sum()
    W = w[0] * np.eye(n)
    for t in range(terms):
        W += w[t + 1] * np.eye(n)[RNG.permutation(n)]
    return W


@pytest.mark.parametrize("topology", ["grid", "expo", "custom"])
def test_gossip_preserves_the_mean_and_contracts_by_beta(topology):
    n, d = 12, 5
    W = _birkhoff(n) if topology == "custom" else None
    Wd = W if W is not None else orc.mixing_matrix(topology, n)
    X = RNG.standard_normal((n, d))
    X1, _ = orc.gossip_pga_step(X, np.zeros_like(X), np.zeros_like(X), 0, topology=topology, H=0, lr=0.1, W=W)
    np.testing.assert_allclose(X1.mean(axis=0), X.mean(axis=0), atol=1e-15)
    np.testing.assert_allclose(X1, Wd @ X, atol=1e-15)
    assert orc.consensus_error(X1) <= orc.beta_of(Wd) * orc.consensus_error(X) + 1e-12   # App. A


def test_custom_W_reproduces_the_named_graphs_and_the_linear_map():
    n, d, lr, mu, H = 6, 3, 0.1, 0.8, 4
    for topology in ("ring", "grid", "expo"):
        W = orc.mixing_matrix(topology, n)
        a = orc.GossipPGA(n, d, topology=topology, H=H, lr=lr, momentum=mu, storage="f64")
        b = orc.GossipPGA(n, d, topology="custom", W=W, H=H, lr=lr, momentum=mu, storage="f64")
        # explicit product form: X_T = sum over steps of (mixing matrices applied to -lr * m)
        Gs = [RNG.standard_normal((n, d)) for _ in range(9)]
        X = np.zeros((n, d))
        M = np.zeros((n, d))
        J = np.full((n, n), 1.0 / n)
        for k, G in enumerate(Gs):
            a.step(G), b.step(G)
            M = mu * M + G
            X = (J if (k + 1) % H == 0 else W) @ (X - lr * M)
            np.testing.assert_allclose(a.X, X, atol=1e-14)
            np.testing.assert_allclose(b.X, X, atol=1e-14)
    with pytest.raises(ValueError):
        orc.GossipPGA(n, d, topology="custom", H=0, lr=0.1)
    with pytest.raises(ValueError):
        orc.GossipPGA(n, d, topology="ring", H=0, lr=0.1, W=np.eye(n))
