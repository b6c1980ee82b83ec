"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
without any reference implementation.  None of these tests needs a GPU."""
import math

import numpy as np
import pytest

from conftest import read_golden
from oracle import gpga_oracle as orc

RNG = np.random.default_rng(12345)


def _J(n):
    return np.full((n, n), 1.0 / n)


# ---------------------------------------------------------------- weight matrix

@pytest.mark.parametrize("topology", ["ring", "expo1", "none", "full"])
@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 20, 32, 100])
def test_W_is_nonnegative_and_doubly_stochastic(topology, n):
    # Sec. 3: W >= 0, W 1 = 1, 1^T W = 1^T, for every iteration's matrix
    for k in range(2 * orc.one_peer_tau(n) + 1):
        W = orc.mixing_matrix(topology, n, k)
        assert (W >= 0).all()
        np.testing.assert_allclose(W.sum(axis=1), 1.0, atol=1e-15)
        np.testing.assert_allclose(W.sum(axis=0), 1.0, atol=1e-15)
        assert (np.diag(W) > 0).all()           # N_i contains i


def test_ring_neighbourhood_is_self_plus_two_with_equal_weights():
    W = orc.mixing_matrix("ring", 8, 0)
    for i in range(8):
        nz = np.nonzero(W[i])[0]
        assert set(nz) == {(i - 1) % 8, i, (i + 1) % 8}      # |N_i| = 3 (Sec. 3.3)
        np.testing.assert_allclose(W[i, nz], 1.0 / 3.0)
    # degenerate sizes fall out of "indices mod n"
    np.testing.assert_allclose(orc.mixing_matrix("ring", 1), [[1.0]])
    np.testing.assert_allclose(orc.mixing_matrix("ring", 2), [[1 / 3, 2 / 3], [2 / 3, 1 / 3]])


def test_ring_beta_matches_values_printed_in_the_paper():
    # Sec. 5.1 prints beta for n = 20, 50, 100 (3 decimals, last one truncated)
    for n_s, beta_s in read_golden("ring_beta.txt"):
        n, printed = int(n_s), float(beta_s)
        beta = orc.beta_of(orc.mixing_matrix("ring", n))
        assert abs(beta - printed) < 1e-3
        # closed form for a symmetric circulant with weights 1/3: second eigenvalue
        assert beta == pytest.approx((1 + 2 * math.cos(2 * math.pi / n)) / 3, abs=1e-12)
    # 1 - beta = O(1/n^2) (Sec. 5.1): quadrupling when n halves
    b1 = 1 - orc.beta_of(orc.mixing_matrix("ring", 64))
    b2 = 1 - orc.beta_of(orc.mixing_matrix("ring", 128))
    assert b1 / b2 == pytest.approx(4.0, rel=2e-3)


def test_ring_eigenvector_is_scaled_by_its_eigenvalue():
    n, q = 12, 2
    v = np.cos(2 * np.pi * q * np.arange(n) / n)[:, None]
    X1, _ = orc.gossip_pga_step(v, np.zeros_like(v), np.zeros_like(v), 0, topology="ring",
                                H=0, lr=0.1, momentum=0.0)
    np.testing.assert_allclose(X1, (1 + 2 * math.cos(2 * math.pi * q / n)) / 3 * v, atol=1e-15)


def test_one_peer_row_i_mixes_with_row_i_plus_power_of_two():
    n = 8
    for k in range(7):
        s = 1 << (k % 3)
        W = orc.mixing_matrix("expo1", n, k)
        for i in range(n):
            assert W[i, i] == 0.5 and W[i, (i + s) % n] == 0.5
            assert np.count_nonzero(W[i]) == 2      # exactly one peer (App. F.1)


@pytest.mark.parametrize("n", [2, 4, 8, 32, 64, 1024])
def test_one_peer_graph_averages_exactly_after_log2_n_gossips(n):
    # Sec. 3: "the exact global average can be achieved via ln(n) gossip communications"
    d = 3
    X = RNG.standard_normal((n, d))
    xbar = X.mean(axis=0)
    Z = np.zeros_like(X)
    for k in range(int(math.log2(n))):
        X, _ = orc.gossip_pga_step(X, Z, Z, k, topology="expo1", H=0, lr=0.3, momentum=0.0)
    np.testing.assert_allclose(X, np.broadcast_to(xbar, X.shape), atol=1e-13)
    # and starting from any phase of the cycle
    X = RNG.standard_normal((n, d))
    xbar = X.mean(axis=0)
    for k in range(5, 5 + int(math.log2(n))):
        X, _ = orc.gossip_pga_step(X, Z, Z, k, topology="expo1", H=0, lr=0.3, momentum=0.0)
    np.testing.assert_allclose(X, np.broadcast_to(xbar, X.shape), atol=1e-13)


@pytest.mark.parametrize("topology", ["ring", "expo1"])
def test_contraction_of_consensus_error_by_beta(topology):
    # App. A: ||(W - J) Y||_F <= beta ||Y||_F ; with G = 0 one gossip step is X <- W X
    n, d = 20, 7
    X = RNG.standard_normal((n, d))
    Z = np.zeros_like(X)
    for k in range(4):
        W = orc.mixing_matrix(topology, n, k)
        X1, _ = orc.gossip_pga_step(X, Z, Z, k, topology=topology, H=0, lr=1.0, momentum=0.0)
        assert orc.consensus_error(X1) <= orc.beta_of(W) * orc.consensus_error(X) * (1 + 1e-12)
        X = X1


# ---------------------------------------------------------------- step structure

def test_schedule_global_average_when_k_plus_1_divisible_by_H():
    assert [k for k in range(12) if orc.is_global_step(k, 4)] == [3, 7, 11]
    assert all(orc.is_global_step(k, 1) for k in range(5))
    assert not any(orc.is_global_step(k, 0) for k in range(100))     # H -> infinity
    # T = 200, H = 4 -> 50 averages, the last step is one
    assert sum(orc.is_global_step(k, 4) for k in range(200)) == 50 and orc.is_global_step(199, 4)


@pytest.mark.parametrize("topology", ["ring", "expo1"])
@pytest.mark.parametrize("momentum", [0.0, 0.9])
def test_gossip_step_preserves_node_mean_of_half_iterate(topology, momentum):
    n, d, lr = 9, 5, 0.07
    X, Mb, G = (RNG.standard_normal((n, d)) for _ in range(3))
    for k in range(4):
        X1, M1 = orc.gossip_pga_step(X, Mb, G, k, topology=topology, H=0, lr=lr, momentum=momentum)
        Y = X - lr * (momentum * Mb + G)            # x^{k+1/2} written out independently
        np.testing.assert_allclose(X1.mean(axis=0), Y.mean(axis=0), atol=1e-14)
        np.testing.assert_allclose(M1, momentum * Mb + G, atol=0)
        # each row is the stated neighbour combination of x^{k+1/2}
        if topology == "ring":
            for i in range(n):
                np.testing.assert_allclose(X1[i], (Y[i - 1] + Y[i] + Y[(i + 1) % n]) / 3, atol=1e-14)
        else:
            s = (1 << (k % 4)) % n
            for i in range(n):
                np.testing.assert_allclose(X1[i], (Y[i] + Y[(i + s) % n]) / 2, atol=1e-14)


def test_global_step_gives_identical_rows_and_zero_consensus_error():
    n, d, lr = 6, 11, 0.2
    X, Mb, G = (RNG.standard_normal((n, d)) for _ in range(3))
    X1, _ = orc.gossip_pga_step(X, Mb, G, 3, topology="ring", H=4, lr=lr, momentum=0.5)
    assert all(np.array_equal(X1[0], X1[i]) for i in range(n))
    # rows are bit-identical; the two-pass fp64 value is 0 up to the rounding of sum/n (n = 6)
    assert orc.consensus_error(X1) <= 1e-16 * np.linalg.norm(X1)
    np.testing.assert_allclose(X1[0], (X - lr * (0.5 * Mb + G)).mean(axis=0), atol=1e-15)


def test_momentum_buffer_is_never_mixed():
    n, d = 5, 3
    X, Mb, G = (RNG.standard_normal((n, d)) for _ in range(3))
    for k, H in ((0, 0), (3, 4)):
        _, M1 = orc.gossip_pga_step(X, Mb, G, k, topology="ring", H=H, lr=0.1, momentum=0.9)
        np.testing.assert_array_equal(M1, 0.9 * Mb + G)


@pytest.mark.parametrize("topology", ["ring", "expo1", "none"])
def test_mean_recursion_holds_on_every_step_type(topology):
    # App. B: xbar^{k+1} = xbar^k - (gamma/n) sum_i g_i, gossip and global steps alike
    n, d, lr, H = 8, 4, 0.05, 3
    sim = orc.GossipPGA(n, d, topology=topology, H=H, lr=lr, momentum=0.0,
                        x0=RNG.standard_normal(d), storage="f64")
    for k in range(10):
        G = RNG.standard_normal((n, d))
        before = sim.X.mean(axis=0)
        sim.step(G)
        np.testing.assert_allclose(sim.X.mean(axis=0), before - lr * G.mean(axis=0), atol=1e-14)


@pytest.mark.parametrize("topology", ["ring", "expo1"])
def test_deviation_closed_form_within_a_period(topology):
    # App. B: X^{k+1} - Xbar^{k+1} = -gamma sum_{l=tau(k)}^{k} prod (W - J) G^{(l)}
    n, d, lr, H = 8, 3, 0.1, 6
    sim = orc.GossipPGA(n, d, topology=topology, H=H, lr=lr, momentum=0.0,
                        x0=RNG.standard_normal(d), storage="f64")
    Gs = []
    J = _J(n)
    for k in range(2 * H - 2):       # crosses one global step, stays inside the 2nd period
        G = RNG.standard_normal((n, d))
        Gs.append(G)
        sim.step(G)
        if orc.is_global_step(k, H):
            assert all(np.array_equal(sim.X[0], sim.X[i]) for i in range(n))
            assert orc.consensus_error(sim.X) <= 1e-15 * np.linalg.norm(sim.X)
            continue
        tau = ((k + 1) // H) * H      # last iterate index at which all rows were equal
        dev = np.zeros((n, d))
        for ell in range(tau, k + 1):
            P = np.eye(n)
            for j in range(ell, k + 1):            # (W_k - J) ... (W_ell - J)
                P = (orc.mixing_matrix(topology, n, j) - J) @ P
            dev -= lr * P @ Gs[ell]
        np.testing.assert_allclose(sim.X - sim.X.mean(axis=0, keepdims=True), dev, atol=1e-13)


@pytest.mark.parametrize("topology", ["ring", "expo1"])
@pytest.mark.parametrize("momentum", [0.0, 0.8])
def test_T_step_map_is_the_explicit_product_of_mixing_matrices(topology, momentum):
    # With prescribed gradients the iteration is linear:
    # X^T = Phi(T,0) X^0 - gamma sum_l Phi(T,l) Mom^l,  Mom^l = sum_{j<=l} mu^{l-j} G^j,
    # Phi(T,l) = A_{T-1} ... A_l with A_k = W_k (gossip) or J (global).
    n, d, lr, H = 6, 2, 0.3, 3
    T = 2 * H + 1
    x0 = RNG.standard_normal(d)
    sim = orc.GossipPGA(n, d, topology=topology, H=H, lr=lr, momentum=momentum, x0=x0, storage="f64")
    Gs = [RNG.standard_normal((n, d)) for _ in range(T)]
    for G in Gs:
        sim.step(G)

    def A(k):
        return _J(n) if (k + 1) % H == 0 else orc.mixing_matrix(topology, n, k)

    def Phi(T_, l):
        P = np.eye(n)
        for k in range(l, T_):
            P = A(k) @ P
        return P

    expect = Phi(T, 0) @ np.tile(x0, (n, 1))
    for l in range(T):
        mom = sum(momentum ** (l - j) * Gs[j] for j in range(l + 1)) if momentum else Gs[l]
        expect = expect - lr * Phi(T, l) @ mom
    np.testing.assert_allclose(sim.X, expect, atol=1e-13)


# ---------------------------------------------------------------- special cases (Sec. 3)

def _tiny_lsq(n=3, d=4, M=8):
    A = RNG.standard_normal((n, M, d))
    b = RNG.standard_normal((n, M))
    return A, b


@pytest.mark.parametrize("momentum", [0.0, 0.7])
def test_H_equal_1_is_parallel_sgd(momentum):
    # Sec. 3: with a global average every step Gossip-PGA is parallel SGD on (1/n) sum f_i
    n, d, M, lr = 3, 4, 8, 0.05
    A, b = _tiny_lsq(n, d, M)
    sim = orc.GossipPGA(n, d, topology="ring", H=1, lr=lr, momentum=momentum, storage="f64")
    x = np.zeros(d)
    v = np.zeros(d)
    for _ in range(25):
        sim.step(orc.lsq_grad(A, b, sim.X))
        # independent centralised loop: full gradient of the average objective
        gbar = np.zeros(d)
        for i in range(n):
            gbar += A[i].T @ (A[i] @ x - b[i]) / M / n
        v = momentum * v + gbar
        x = x - lr * v
        np.testing.assert_allclose(sim.X, np.tile(x, (n, 1)), atol=1e-13)


def test_topology_full_equals_H_equal_1():
    n, d = 5, 3
    a = orc.GossipPGA(n, d, topology="full", H=0, lr=0.1, momentum=0.0, storage="f64")
    b = orc.GossipPGA(n, d, topology="ring", H=1, lr=0.1, momentum=0.0, storage="f64")
    for _ in range(4):
        G = RNG.standard_normal((n, d))
        a.step(G), b.step(G)
        np.testing.assert_allclose(a.X, b.X, atol=1e-15)


def test_W_identity_is_local_sgd_and_H_infinite_is_gossip_sgd():
    n, d, lr, H = 4, 3, 0.1, 5
    loc = orc.GossipPGA(n, d, topology="none", H=H, lr=lr, storage="f64")
    gos = orc.GossipPGA(n, d, topology="ring", H=0, lr=lr, storage="f64")
    xs = np.zeros((n, d))                 # independent Local SGD: nodes never talk between averages
    xg = np.zeros((n, d))
    W = orc.mixing_matrix("ring", n)
    for k in range(12):
        G = RNG.standard_normal((n, d))
        loc.step(G), gos.step(G)
        xs = xs - lr * G
        if (k + 1) % H == 0:
            xs[:] = xs.mean(axis=0)
        xg = W @ (xg - lr * G)
        np.testing.assert_allclose(loc.X, xs, atol=1e-14)
        np.testing.assert_allclose(gos.X, xg, atol=1e-14)


def test_least_squares_reaches_the_normal_equation_solution():
    n, d, M = 3, 4, 8
    A, b = _tiny_lsq(n, d, M)
    sim = orc.GossipPGA(n, d, topology="ring", H=1, lr=0.1, momentum=0.0, storage="f64")
    # one step by hand
    g0 = np.stack([A[i].T @ (A[i] @ np.zeros(d) - b[i]) / M for i in range(n)])
    sim.step(orc.lsq_grad(A, b, sim.X))
    np.testing.assert_allclose(sim.X[0], -0.1 * g0.mean(axis=0), atol=1e-15)
    for _ in range(3000):
        sim.step(orc.lsq_grad(A, b, sim.X))
    sol = np.linalg.lstsq(A.reshape(n * M, d), b.reshape(n * M), rcond=None)[0]
    np.testing.assert_allclose(sim.X[1], sol, atol=1e-9)


def test_gossip_pga_with_gossip_steps_also_converges_near_least_squares_solution():
    # decentralised run (ring, H=4): node mean approaches the same minimiser
    n, d, M = 4, 3, 10
    A, b = _tiny_lsq(n, d, M)
    sim = orc.GossipPGA(n, d, topology="ring", H=4, lr=0.02, momentum=0.0, storage="f64")
    for _ in range(6000):
        sim.step(orc.lsq_grad(A, b, sim.X))
    sol = np.linalg.lstsq(A.reshape(n * M, d), b.reshape(n * M), rcond=None)[0]
    # constant step + heterogeneous data leaves an O(gamma) bias, not an exact fixed point
    assert np.linalg.norm(sim.X.mean(axis=0) - sol) < 0.05 * max(1.0, np.linalg.norm(sol))


# ---------------------------------------------------------------- gradients

def _fd(loss, X, i, eps=1e-6):
    g = np.zeros(X.shape[1])
    for c in range(X.shape[1]):
        Xp, Xm = X.copy(), X.copy()
        Xp[i, c] += eps
        Xm[i, c] -= eps
        g[c] = (loss(Xp)[i] - loss(Xm)[i]) / (2 * eps)
    return g


@pytest.mark.parametrize("use_idx", [False, True])
def test_gradients_match_central_finite_differences(use_idx):
    n, d, M = 3, 5, 7
    A = RNG.standard_normal((n, M, d))
    b = RNG.standard_normal((n, M))
    y = np.where(RNG.random((n, M)) < 0.5, 1.0, -1.0)
    X = RNG.standard_normal((n, d))
    idx = RNG.integers(0, M, size=(n, 4)) if use_idx else None
    G_ls = orc.lsq_grad(A, b, X, idx)
    G_lr = orc.logreg_grad(A, y, X, idx)
    for i in range(n):
        np.testing.assert_allclose(G_ls[i], _fd(lambda Z: orc.lsq_loss(A, b, Z, idx), X, i), atol=1e-7)
        np.testing.assert_allclose(G_lr[i], _fd(lambda Z: orc.logreg_loss(A, y, Z, idx), X, i), atol=1e-7)


def test_logistic_loss_is_the_papers_formula_and_stable_for_large_margins():
    # Sec. 5.1: f_i(x) = (1/M) sum ln(1 + exp(-y h^T x))
    h = np.array([[[1.0, 2.0], [3.0, -1.0]]])
    y = np.array([[1.0, -1.0]])
    x = np.array([[0.5, -0.25]])
    want = 0.5 * (math.log(1 + math.exp(-(0.5 - 0.5))) + math.log(1 + math.exp(+(1.5 + 0.25))))
    assert orc.logreg_loss(h, y, x)[0] == pytest.approx(want, rel=1e-14)
    big = orc.logreg_loss(h * 1e4, y, x)
    assert np.isfinite(big).all()
    assert np.isfinite(orc.logreg_grad(h * 1e4, y, x)).all()


def test_gradient_uses_each_nodes_own_iterate_and_own_data():
    n, d, M = 3, 4, 6
    A = RNG.standard_normal((n, M, d))
    b = RNG.standard_normal((n, M))
    X = RNG.standard_normal((n, d))
    G = orc.lsq_grad(A, b, X)
    X2 = X.copy()
    X2[1] += 1.0
    G2 = orc.lsq_grad(A, b, X2)
    assert np.array_equal(G[0], G2[0]) and np.array_equal(G[2], G2[2]) and not np.array_equal(G[1], G2[1])


# ---------------------------------------------------------------- counter RNG

def test_philox_known_answer_vectors():
    for row in read_golden("philox4x32_10_kat.txt"):
        w = [int(t, 16) for t in row]
        out = orc.philox4x32_10(w[0], w[1], w[2], w[3], w[4], w[5])
        assert [int(o) for o in out] == w[6:10]


def test_philox_is_vectorised_consistently():
    c0 = np.arange(17, dtype=np.uint64)
    out = orc.philox4x32_10(c0, 5, 9, 1, 0xDEADBEEF, 0x1234)
    for j in range(17):
        one = orc.philox4x32_10(j, 5, 9, 1, 0xDEADBEEF, 0x1234)
        assert [int(o[j]) for o in out] == [int(o) for o in one]


def test_uniform_mapping_is_open_interval_and_exact_in_fp32():
    u = orc._uniform23(np.array([0, 511, 512, 0xFFFFFFFF], dtype=np.uint64))
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24 and u[2] == 1.5 * 2.0 ** -23
    assert u[3] == 1.0 - 2.0 ** -24 and (u > 0).all() and (u < 1).all()
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)


def test_counter_normals_have_standard_moments_and_independent_lanes():
    z = orc.counter_normals(7, orc.TAG_GRAD, 3, 11, np.arange(250_000))      # (250000, 4)
    flat = z.ravel()
    N = flat.size
    assert abs(flat.mean()) < 5 / math.sqrt(N)
    assert abs(flat.var() - 1.0) < 5 * math.sqrt(2.0 / N)
    assert abs((flat ** 4).mean() - 3.0) < 5 * math.sqrt(96.0 / N)
    assert abs((flat ** 3).mean()) < 5 * math.sqrt(15.0 / N)
    C = np.corrcoef(z.T)
    assert np.abs(C - np.eye(4)).max() < 5 / math.sqrt(z.shape[0])
    # tail mass beyond 3 sigma ~ 0.0027
    assert abs((np.abs(flat) > 3).mean() - 0.0026998) < 5 * math.sqrt(0.0027 / N)


def test_box_muller_pairs_invert_to_their_own_uniform_words():
    # Box-Muller read backwards: the squared radius of a pair is -2 ln u_a and its angle
    # 2 pi u_b, with (u_a, u_b) from words (r0, r1) for columns 0, 1 and (r2, r3) for columns
    # 2, 3 of a quad.  The words come from the generator pinned by the known-answer vectors.
    seed, node, j = 0x1234567890, 5, 9
    c4 = np.arange(4096)
    z = orc.counter_normals(seed, orc.TAG_FEAT, node, j, c4)
    r = orc.philox4x32_10(c4, node, j, orc.TAG_FEAT, seed & 0xFFFFFFFF, seed >> 32)
    u = [((np.asarray(w, dtype=np.uint64) >> np.uint64(9)).astype(np.float64) + 0.5) / 2.0 ** 23 for w in r]
    for pair, (ua, ub) in enumerate(((u[0], u[1]), (u[2], u[3]))):
        a, b = z[:, 2 * pair], z[:, 2 * pair + 1]
        np.testing.assert_allclose(np.exp(-0.5 * (a * a + b * b)), ua, rtol=1e-12)
        turn = np.mod(np.arctan2(b, a) / (2.0 * np.pi), 1.0)
        gap = np.abs(turn - ub)
        assert np.minimum(gap, 1.0 - gap).max() < 1e-12
    # the two pairs of a quad are independent draws: their squared radii are uncorrelated
    z = orc.counter_normals(7, orc.TAG_GRAD, 3, 11, np.arange(100_000))
    ra2, rb2 = z[:, 0] ** 2 + z[:, 1] ** 2, z[:, 2] ** 2 + z[:, 3] ** 2
    assert abs(np.corrcoef(ra2, rb2)[0, 1]) < 5 / math.sqrt(len(ra2))


def test_synthetic_gradient_addressing_and_variance():
    n, var = 4, 1e-3
    full = orc.synthetic_grad(0, 5, n, np.arange(64), var)
    some = orc.synthetic_grad(0, 5, n, np.array([3, 4, 17, 62, 63]), var)
    np.testing.assert_array_equal(some, full[:, [3, 4, 17, 62, 63]])
    assert not np.array_equal(full, orc.synthetic_grad(0, 6, n, np.arange(64), var))   # new k, new draw
    assert not np.array_equal(full[0], full[1])                                        # per node
    assert not np.array_equal(full, orc.synthetic_grad(1, 5, n, np.arange(64), var))   # seed
    big = orc.synthetic_grad(0, 0, 8, np.arange(100_000), var)
    assert abs(big.var() / var - 1.0) < 0.01           # N(0, var): var is a variance


def test_virtual_feature_gradient_equals_gradient_on_materialised_features():
    n, d, M, B, seed, mu_var = 3, 40, 6, 4, 3, 0.5
    X = RNG.standard_normal((n, d))
    y = np.where(RNG.random((n, M)) < 0.5, 1.0, -1.0)
    idx = RNG.integers(0, M, size=(n, B))
    feat = np.stack([orc.virtual_features(seed, i, np.arange(M), np.arange(d), mu_var) for i in range(n)])
    feat = feat.astype(np.float32)
    G1 = orc.logreg_virtual_grad(seed, y, X, idx, mu_var, chunk=16)
    G2 = orc.logreg_grad(feat, y, X, idx)
    np.testing.assert_allclose(G1, G2, atol=1e-13)
    # the node shift is a draw of its own: uncorrelated with the noise of any sample
    cols = np.arange(20_000)
    mu = orc.virtual_features(seed, 1, np.arange(3000), cols[:50], mu_var).mean(axis=0)   # ~ mu_1[:50]
    shift = orc.virtual_features(seed, 1, [0], cols, 1.0)[0] - orc.virtual_features(seed, 1, [0], cols, 0.0)[0]
    np.testing.assert_allclose(shift[:50] * math.sqrt(mu_var), mu, atol=5 / math.sqrt(3000))
    for m in range(4):
        zeta = orc.virtual_features(seed, 1, [m], cols, 0.0)[0]
        assert abs(np.corrcoef(shift, zeta)[0, 1]) < 5 / math.sqrt(len(cols))
    # node shift: sample mean over many samples approaches mu_i, with variance mu_var across columns
    cols = np.arange(2000)
    h = orc.virtual_features(seed, 1, np.arange(400), cols, mu_var)
    mu_hat = h.mean(axis=0)
    assert abs(mu_hat.var() - mu_var) < 0.08
    assert abs((h - mu_hat).var() - 1.0) < 0.02


# ---------------------------------------------------------------- reductions

def test_consensus_error_equals_norm_of_I_minus_J_times_X():
    n, d = 7, 5
    X = RNG.standard_normal((n, d))
    want = np.linalg.norm((np.eye(n) - _J(n)) @ X, "fro")
    assert orc.consensus_error(X) == pytest.approx(want, rel=1e-14)
    np.testing.assert_allclose(orc.node_mean(X), np.ones(n) @ X / n, atol=1e-15)
    assert orc.consensus_error(np.tile(X[0], (n, 1))) <= 1e-15 * np.linalg.norm(X[0])


def test_fp32_storage_mode_rounds_state_only_between_steps():
    n, d = 4, 6
    a = orc.GossipPGA(n, d, topology="ring", H=3, lr=0.1, momentum=0.9, storage="f32")
    b = orc.GossipPGA(n, d, topology="ring", H=3, lr=0.1, momentum=0.9, storage="f64")
    for _ in range(7):
        G = RNG.standard_normal((n, d))
        a.step(G), b.step(G)
        assert np.array_equal(a.X, a.X.astype(np.float32).astype(np.float64))
        assert np.array_equal(a.M, a.M.astype(np.float32).astype(np.float64))
    np.testing.assert_allclose(a.X, b.X, rtol=0, atol=1e-5)
    assert not np.array_equal(a.X, b.X)


# ---------------------------------------------------------------- adaptive period (Algorithm 2)

def test_aga_period_schedule_on_a_hand_worked_example():
    # H_init = 2, K_w = 4, losses identical on all nodes: F_k = 8 / (k + 1).
    # k=1: C hits 2 -> average; k < 4: F_init = (0 + 4)/2 = 2
    # k=3: average; k < 4: F_init = (2 + 2)/2 = 2
    # k=5: average; F = 8/6:   H = ceil(2 / (8/6) * 2)  = ceil(3)   = 3
    # k=8: average; F = 8/9:   H = ceil(2 / (8/9) * 2)  = ceil(4.5) = 5
    # k=13: average; F = 8/14: H = ceil(2 / (8/14) * 2) = ceil(7)   = 7
    # k=20: average; F = 8/21: H = ceil(10.5) = 11 -> capped at H_max = 9
    n, d = 4, 3
    sim = orc.GossipAGA(n, d, topology="ring", H_init=2, warmup_iters=4, H_max=9, lr=0.1, storage="f64")
    averaged_at = []
    for k in range(24):
        G = RNG.standard_normal((n, d))
        sim.step(G, np.full(n, 8.0 / (k + 1)))
        rows_equal = all(np.array_equal(sim.X[0], sim.X[i]) for i in range(n))
        if rows_equal:
            averaged_at.append(k)
    assert averaged_at == [1, 3, 5, 8, 13, 20]
    assert sim.history == [(1, 2), (3, 2), (5, 3), (8, 5), (13, 7), (20, 9)]
    assert sim.F_init == 2.0


def test_aga_warm_up_ends_with_iteration_K_w_itself():
    # Algorithm 2 tests k < K_w: an average that falls on k = K_w already adapts the period
    n, d = 3, 2
    sim = orc.GossipAGA(n, d, topology="ring", H_init=2, warmup_iters=3, H_max=10, lr=0.1, storage="f64")
    Z = np.zeros((n, d))
    for k in range(4):
        sim.step(Z, np.full(n, 4.0))
    # k=1: warm-up, F_init = (0 + 4)/2 = 2;  k=3 = K_w: H = ceil(2 / 4 * 2) = 1, F_init untouched
    assert sim.history == [(1, 2), (3, 1)] and sim.F_init == 2.0


def test_aga_with_constant_period_is_gossip_pga():
    # losses chosen so that ceil(F_init / F * H_init) stays H_init: the counter schedule
    # then averages exactly when mod(k+1, H) = 0, i.e. Algorithm 1
    n, d, H = 6, 4, 3
    def lr(k):                                            # a schedule: both must read gamma_k at the same k
        return 0.05 * 0.9 ** k
    aga = orc.GossipAGA(n, d, topology="expo1", H_init=H, warmup_iters=7, H_max=50, lr=lr, momentum=0.9,
                        storage="f64")
    pga = orc.GossipPGA(n, d, topology="expo1", H=H, lr=lr, momentum=0.9, storage="f64")
    for k in range(20):
        G = RNG.standard_normal((n, d))
        # warm-up (k = 2, 5 < 7) sees F = 4, 4: F_init = 2, then 3; afterwards F = 3.2 gives
        # ceil(3 / 3.2 * 3) = ceil(2.8125) = 3
        aga.step(G, np.full(n, 4.0 if k < 7 else 3.2))
        pga.step(G)
        np.testing.assert_allclose(aga.X, pga.X, atol=1e-15)
        np.testing.assert_allclose(aga.M, pga.M, atol=1e-15)
    assert aga.F_init == 3.0 and aga.H == H


def test_aga_uses_the_node_mean_of_the_losses_and_clamps_the_period():
    n, d = 5, 2
    sim = orc.GossipAGA(n, d, topology="ring", H_init=2, warmup_iters=2, H_max=6, lr=0.1, storage="f64")
    Z = np.zeros((n, d))
    sim.step(Z, np.arange(n, dtype=float))            # k=0: C=1
    sim.step(Z, np.array([1.0, 2.0, 3.0, 4.0, 10.0]))  # k=1: average, warm-up: F = 4 -> F_init = 2
    assert sim.F_init == 2.0
    sim.step(Z, np.ones(n))
    sim.step(Z, np.array([0.5, 0.5, 0.5, 0.5, 0.5]))   # k=3: F = 0.5 -> ceil(2/0.5*2) = 8 -> clamp 6
    assert sim.H == 6
    for _ in range(6):
        sim.step(Z, np.full(n, 100.0))                 # next average at k=9: ceil(2/100*2) = 1
    assert sim.H == 1 and sim.history[-1] == (9, 1)
    sim.step(Z, np.zeros(n))                           # F = 0: period goes to H_max
    assert sim.H == 6
