"""GPU parity of gossip steps with a sparse weight matrix (grid, static
exponential graph, caller-supplied W) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import gpga_oracle as orc
from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_STEP = 1e-5
TOL_FINAL = 1e-4


@pytest.fixture(scope="module")
def hx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import harness
    return harness


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return (np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300),
            np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def assert_close(got, ref, tol, what=""):
    emax, efro = rel_errors(got, ref)
    assert emax <= tol and efro <= tol, f"{what}: max-rel {emax:.3e}, fro-rel {efro:.3e} > {tol:g}"


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def birkhoff(n, seed, terms=4):
    """Random doubly stochastic W: convex combination of permutation matrices (plus I)."""
    rng = np.random.default_rng(seed)
    w = rng.random(terms + 1)
    w /= w.sum()
    W = w[0] * np.eye(n)
    for t in range(terms):
        W += w[t + 1] * np.eye(n)[rng.permutation(n)]
    return W.astype(np.float32).astype(np.float64)      # the values the library will hold


CASES = [
    # n, d, ld_pad, topology, momentum, nesterov, H, k
    (2, 7, 0, "grid", 0.0, False, 0, 0),
    (3, 256, 0, "expo", 0.9, False, 0, 1),
    (4, 300, 0, "grid", 0.9, False, 0, 0),              # 2 x 2: folded neighbours
    (7, 301, 0, "grid", 0.5, False, 0, 2),              # prime n: 1 x 7
    (12, 1031, 1, "grid", 0.9, False, 0, 5),            # vector path plus 3-column tail
    (12, 1030, 2, "expo", 0.9, False, 0, 5),            # scalar path
    (20, 515, 1, "grid", 0.9, True, 16, 3),
    (20, 515, 1, "grid", 0.9, True, 16, 15),            # global average
    (64, 4100, 0, "grid", 0.9, False, 48, 7),           # 8 x 8, 16-byte lanes, a 64 KiB tile
    (64, 4100, 0, "expo", 0.9, False, 48, 7),
    (64, 40_000, 0, "expo", 0.0, False, 0, 0),
    (65, 2052, 0, "grid", 0.9, False, 0, 1),            # 8-byte lanes
    (100, 2052, 0, "expo", 0.9, True, 0, 1),
    (128, 1000, 0, "grid", 0.9, False, 0, 0),
    (129, 1000, 0, "grid", 0.9, False, 0, 0),           # 4-byte lanes
    (256, 777, 0, "expo", 0.9, False, 0, 0),
    (257, 777, 0, "grid", 0.9, False, 0, 0),            # two-pass path
    (1024, 2052, 0, "grid", 0.9, False, 8, 0),          # 32 x 32, two-pass
    (1024, 2051, 0, "expo", 0.9, True, 8, 3),
    (1024, 520, 0, "grid", 0.9, False, 8, 7),           # global average
    (9, 500, 0, "custom", 0.9, False, 0, 0),
    (64, 4100, 0, "custom", 0.9, True, 0, 3),
    (300, 1028, 0, "custom", 0.0, False, 0, 0),
]


@pytest.mark.parametrize("n,d,pad,topology,momentum,nesterov,H,k", CASES)
def test_sparse_W_step_matches_oracle(hx, n, d, pad, topology, momentum, nesterov, H, k):
    X, Mb, G = inputs.random_state(n, d, seed=7000 + n + d + k)
    lr = 0.37
    W = birkhoff(n, seed=n) if topology == "custom" else None
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=lr, momentum=momentum, ld=d + pad)
    if W is not None:
        sim.set_mixing(W)
    if nesterov:
        sim.set_nesterov(True)
    sim.set_state(X=X, M=Mb, G=G, k=k)
    sim.step()
    X_ref, M_ref = orc.gossip_pga_step(X, Mb if momentum else np.zeros_like(Mb), G, k, topology=topology, H=H,
                                       lr=lr, momentum=momentum, nesterov=nesterov, W=W)
    assert sim.k == k + 1
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    if momentum:
        assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    if orc.is_global_step(k, H):
        Xg = sim.X.cpu().numpy()
        assert all(np.array_equal(Xg[0], Xg[i]) for i in range(n))
    sim.close()


@pytest.mark.parametrize("n,d,topology", [(20, 1031, "grid"), (64, 4100, "expo"), (100, 515, "grid")])
def test_two_pass_path_gives_the_tile_kernels_answer_and_leaves_g_alone(hx, n, d, topology):
    X, Mb, G = inputs.random_state(n, d, seed=31 + n)
    outs = []
    for two_pass in (0, 1):
        sim = hx.Simulation(n, d, topology=topology, H=0, lr=0.1, momentum=0.9)
        sim.set_option("mix_two_pass", two_pass)
        sim.set_state(X=X, M=Mb, G=G, k=0)
        sim.step()
        assert int(sim.query("step_path")) == (6 if two_pass else 4)
        outs.append((host(sim.X), host(sim.M), host(sim.G)))
        sim.close()
    X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, 0, topology=topology, H=0, lr=0.1, momentum=0.9)
    for Xg, Mg, Gg in outs:
        assert_close(Xg, X_ref, TOL_STEP, "X")
        assert_close(Mg, M_ref, TOL_STEP, "M")
        np.testing.assert_array_equal(Gg, G)             # both paths leave the gradients as they were


@pytest.mark.parametrize("opts", [{"blocks_per_cu": 1}, {"blocks_per_cu": 1, "pace_gbs": 3000},
                                  {"blocks_per_cu": 2, "pace_gbs": 8000, "mix_waves": 4}, {"mix_waves": 16},
                                  {"mix_lane_bytes": 8}, {"mix_lane_bytes": 4, "mix_waves": 2}, {"mix_csr_lds": 0},
                                  {"mix_csr_lds": 0, "mix_lane_bytes": 8, "mix_waves": 4}],
                         ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
@pytest.mark.parametrize("topology", ["grid", "expo"])
def test_tile_kernel_launch_shapes_give_the_same_answer(hx, topology, opts):
    # wide enough that a capped grid strides over several tiles per workgroup (and waits on its deadlines)
    n, d = 64, 300_004
    X, Mb, G = inputs.random_state(n, d, seed=77)
    sim = hx.Simulation(n, d, topology=topology, H=0, lr=0.1, momentum=0.9)
    for name, v in opts.items():
        sim.set_option(name, v)
    sim.set_state(X=X, M=Mb, G=G, k=0)
    X_ref, M_ref = X, Mb
    for j in range(2):
        sim.step()
        X_ref, M_ref = orc.gossip_pga_step(X_ref, M_ref, G, j, topology=topology, H=0, lr=0.1, momentum=0.9)
        X_ref = X_ref.astype(np.float32).astype(np.float64)
        M_ref = M_ref.astype(np.float32).astype(np.float64)
        assert_close(host(sim.X), X_ref, TOL_STEP, f"X after step {j}")
        assert_close(host(sim.M), M_ref, TOL_STEP, f"M after step {j}")
    sim.close()


def test_custom_W_equal_to_the_ring_matches_the_ring_stencil_kernel(hx):
    n, d = 64, 5000
    X, Mb, G = inputs.random_state(n, d, seed=3)
    a = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.9)
    b = hx.Simulation(n, d, topology="custom", H=0, lr=0.1, momentum=0.9)
    b.set_mixing(orc.mixing_matrix("ring", n))
    for sim in (a, b):
        sim.set_state(X=X, M=Mb, G=G, k=0)
        sim.step()
    assert_close(host(b.X), host(a.X), 1e-6, "custom ring vs stencil ring")
    assert a.beta == pytest.approx(b.beta, abs=1e-7)
    assert a.beta == pytest.approx(orc.beta_of(orc.mixing_matrix("ring", n)), abs=2e-7)
    a.close(), b.close()


def test_custom_topology_without_a_matrix_is_a_state_error_and_bad_W_is_rejected(hx):
    from paper_2105_09080_amd import binding as B
    n, d = 6, 64
    sim = hx.Simulation(n, d, topology="custom", H=0, lr=0.1, momentum=0.0)
    with pytest.raises(B.GpgaError) as e:
        sim.step()
    assert e.value.status == B.GPGA_ESTATE
    with pytest.raises(B.GpgaError) as e:
        _ = sim.beta
    assert e.value.status == B.GPGA_ESTATE
    W = np.full((n, n), 1.0 / n)
    W[0, 0] += 0.01                                       # not stochastic any more
    with pytest.raises(B.GpgaError) as e:
        sim.set_mixing(W)
    assert e.value.status == B.GPGA_EINVAL
    sim.set_mixing(np.full((n, n), 1.0 / n))              # dense J is a valid W
    X, _, G = inputs.random_state(n, d, seed=1)
    sim.set_state(X=X, G=G, k=0)
    sim.step()
    X_ref, _ = orc.gossip_pga_step(X, np.zeros_like(X), G, 0, topology="full", H=0, lr=0.1)
    assert_close(host(sim.X), X_ref, TOL_STEP, "W = J through the sparse path")
    assert sim.beta == pytest.approx(0.0, abs=1e-6)
    sim.close()


@pytest.mark.parametrize("topology", ["grid", "expo"])
def test_logistic_trajectory_on_the_appendix_topologies(hx, topology):
    # shape family of the appendix experiments (App. F.2): logistic regression, non-iid nodes,
    # n = 20, H = 16; features scaled so that the free-running comparison is meaningful
    n, d, M, Bsz, T, H = 20, 1000, 60, 8, 120, 16
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=11, mu_var=0.5, label_noise_std=0.1)
    feat = (feat / np.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, Bsz, M, seed=11)
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.2, momentum=0.9)
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(idx)
    ref = orc.GossipPGA(n, d, topology=topology, H=H, lr=float(np.float32(0.2)), momentum=0.9, storage="f32")
    cons = []
    for k in range(T):
        sim.local_grad(idx_d[k])
        sim.step()
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]))
        ce, ce_ref = sim.consensus_error(), orc.consensus_error(ref.X)
        assert abs(ce - ce_ref) <= 1e-4 * max(ce_ref, 1e-3 * np.linalg.norm(ref.X)), (k, ce, ce_ref)
        cons.append(ce)
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    assert all(cons[k] <= 1e-6 * np.linalg.norm(ref.X) for k in range(H - 1, T, H))   # zero right after each average
    sim.close()


def banded(n, band, seed):
    """Random doubly stochastic W whose neighbours all lie within circular distance `band`:
    a convex combination of cyclic shifts by -band .. band (a circulant; every shift is a permutation)."""
    rng = np.random.default_rng(seed)
    shifts = np.arange(-band, band + 1)
    w = rng.random(len(shifts)) * (rng.random(len(shifts)) < 0.7)
    w[band] += 0.2                        # self weight
    w[0] += 0.05                          # keep the band as wide as asked for
    w /= w.sum()
    W = sum(wk * np.roll(np.eye(n), s, axis=1) for wk, s in zip(w, shifts))
    return W.astype(np.float32).astype(np.float64)


BAND_CASES = [
    # n, d, ld_pad, topology (or band of a custom circulant), momentum, nesterov
    (20, 515, 1, "grid", 0.9, False),            # 4 x 5 torus: band 5 = n / 4, vector path plus a tail
    (25, 300, 0, "grid", 0.0, False),            # 5 x 5
    (64, 4100, 0, "grid", 0.9, False),           # 8 x 8, 16-byte lanes
    (64, 4102, 2, "grid", 0.9, True),            # rows not 16-byte aligned: 4-byte lanes
    (100, 2052, 0, "grid", 0.9, True),           # 10 x 10
    (256, 1000, 0, "grid", 0.9, False),          # 16 x 16
    (1024, 2052, 0, "grid", 0.9, False),         # 32 x 32: band 32, the kept rows and the ring hold 144 rows
    (1023, 700, 0, 31, 0.5, False),              # n not a multiple of the wavefronts per workgroup
    (992, 516, 0, "grid", 0.9, False),           # 31 x 32
    (37, 900, 0, 1, 0.9, False),                 # a ring with random weights
    (50, 1234, 0, 3, 0.9, False),
    (333, 640, 0, 7, 0.9, True),
    (2000, 260, 0, 32, 0.0, False),              # the widest band the kernel takes
]


@pytest.mark.parametrize("n,d,pad,topology,momentum,nesterov", BAND_CASES)
def test_banded_W_sliding_window_kernel_matches_oracle(hx, n, d, pad, topology, momentum, nesterov):
    X, Mb, G = inputs.random_state(n, d, seed=9000 + n + d)
    lr = 0.37
    W = banded(n, topology, seed=n) if isinstance(topology, int) else None
    name = "custom" if W is not None else topology
    sim = hx.Simulation(n, d, topology=name, H=0, lr=lr, momentum=momentum, ld=d + pad)
    if W is not None:
        sim.set_mixing(W)
    if nesterov:
        sim.set_nesterov(True)
    sim.set_option("mix_band", 1)
    X_ref, M_ref = X, (Mb if momentum else np.zeros_like(Mb))
    sim.set_state(X=X, M=Mb, G=G, k=0)
    for k in range(2):          # two steps: both directions of the ping-pong
        sim.step()
        assert int(sim.query("step_path")) == 5, "the sliding-window kernel did not take this W"
        X_ref, M_ref = orc.gossip_pga_step(X_ref, M_ref, G, k, topology=name, H=0, lr=lr, momentum=momentum,
                                           nesterov=nesterov, W=W)
        X_ref = X_ref.astype(np.float32).astype(np.float64)
        M_ref = M_ref.astype(np.float32).astype(np.float64)
        assert_close(host(sim.X), X_ref, TOL_STEP, f"X after step {k}")
        if momentum:
            assert_close(host(sim.M), M_ref, TOL_STEP, f"M after step {k}")
    np.testing.assert_array_equal(host(sim.G), G.astype(np.float64))      # the gradients are only read
    sim.close()


def test_a_band_wider_than_the_kernel_takes_falls_back_to_two_passes(hx):
    n, d = 1023, 700             # 31 x 33 torus: neighbours 33 rows away, one more than the sliding window holds
    X, Mb, G = inputs.random_state(n, d, seed=5)
    sim = hx.Simulation(n, d, topology="grid", H=0, lr=0.1, momentum=0.5)
    sim.set_option("mix_band", 1)
    sim.set_state(X=X, M=Mb, G=G, k=0)
    sim.step()
    assert int(sim.query("step_path")) == 6
    X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, 0, topology="grid", H=0, lr=0.1, momentum=0.5)
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    sim.close()


@pytest.mark.parametrize("opts", [{"blocks_per_cu": 1}, {"blocks_per_cu": 2, "pace_gbs": 3000}, {"mix_lane_bytes": 8},
                                  {"mix_lane_bytes": 4, "pace_gbs": 8000}],
                         ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
def test_banded_kernel_persistent_and_paced(hx, opts):
    n, d = 64, 300_004          # more column tiles than resident workgroups
    X, Mb, G = inputs.random_state(n, d, seed=77)
    sim = hx.Simulation(n, d, topology="grid", H=0, lr=0.1, momentum=0.9)
    sim.set_option("mix_band", 1)
    for name, v in opts.items():
        sim.set_option(name, v)
    sim.set_state(X=X, M=Mb, G=G, k=0)
    sim.step()
    assert int(sim.query("step_path")) == 5
    assert int(sim.query("step_paced")) == (1 if "pace_gbs" in opts else 0)
    assert int(sim.query("step_lane_bytes")) == opts.get("mix_lane_bytes", 16)
    X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, 0, topology="grid", H=0, lr=0.1, momentum=0.9)
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    sim.close()
