"""GPU parity: every entry point of libgpga, called through the C ABI, compared
element by element with the CPU oracle on the same seeded inputs.

Tolerances (fp32 arithmetic against a float64 oracle):
  TOL_STEP  = 1e-5   one call of an entry point on identical inputs
  TOL_FINAL = 1e-4   final iterates of a free-running trajectory
both as max|diff| / max|reference| and as ||diff||_F / ||reference||_F.
"""
import math

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
    scale_max = max(np.abs(ref).max(), 1e-300)
    scale_f = max(np.linalg.norm(ref), 1e-300)
    return np.abs(got - ref).max() / scale_max, np.linalg.norm(got - ref) / scale_f


def assert_close(got, ref, tol, what=""):
    emax, efro = rel_errors(got, ref)
    assert emax <= tol and efro <= tol, f"{what}: max-rel {emax:.3e}, fro-rel {efro:.3e} > {tol:g}"


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


# ------------------------------------------------------------------ one fused step

STEP_CASES = [
    # n, d, ld_pad, topology, momentum, H, k
    (1, 5, 0, "ring", 0.9, 0, 0),
    (2, 7, 0, "ring", 0.0, 0, 0),
    (3, 256, 0, "ring", 0.9, 0, 1),
    (8, 1000, 0, "ring", 0.0, 4, 0),
    (8, 1000, 0, "ring", 0.0, 4, 3),          # global
    (8, 1030, 2, "ring", 0.9, 0, 5),          # ragged d, padded unaligned ld -> scalar path
    (8, 1031, 1, "ring", 0.9, 0, 5),          # vector path plus 3-column tail
    (64, 4100, 0, "ring", 0.9, 48, 7),
    (64, 4100, 0, "ring", 0.9, 48, 47),       # global
    (100, 515, 1, "ring", 0.5, 0, 2),
    (1, 9, 0, "expo1", 0.9, 0, 3),
    (2, 64, 0, "expo1", 0.9, 0, 1),
    (6, 300, 0, "expo1", 0.9, 0, 2),          # non power of two: offset 4, two cycles of 3
    (7, 300, 0, "expo1", 0.0, 0, 1),
    (32, 10000, 0, "expo1", 0.9, 16, 0),
    (32, 10000, 0, "expo1", 0.9, 16, 3),
    (32, 10000, 0, "expo1", 0.9, 16, 4),      # offset 16: cycles of two rows
    (32, 10000, 0, "expo1", 0.9, 16, 15),     # global
    (64, 2052, 0, "expo1", 0.9, 6, 2),
    (64, 2052, 4, "expo1", 0.9, 6, 4),
    (1024, 520, 0, "ring", 0.9, 8, 0),
    (1024, 520, 0, "ring", 0.9, 8, 7),        # global, many rows
    (1024, 520, 0, "expo1", 0.9, 0, 9),       # offset 512
    (1024, 520, 0, "expo1", 0.9, 0, 3),
    (16, 777, 0, "none", 0.9, 5, 1),
    (16, 777, 0, "none", 0.9, 5, 4),          # global
    (16, 777, 0, "full", 0.3, 0, 1),          # W = J: every step is global
]


@pytest.mark.parametrize("n,d,pad,topology,momentum,H,k", STEP_CASES)
def test_single_step_matches_oracle(hx, n, d, pad, topology, momentum, H, k):
    X, Mb, G = inputs.random_state(n, d, seed=1000 + n + d + k)
    lr = 0.37
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=lr, momentum=momentum, ld=d + pad)
    sim.set_state(X=X, M=Mb, G=G, k=k)
    sim.step()
    X_ref, M_ref = orc.gossip_pga_step(X, Mb if momentum else np.zeros_like(Mb), G, k, topology=topology,
                                       H=H, lr=lr, momentum=momentum)
    assert sim.k == k + 1
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    if momentum:
        assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    if orc.is_global_step(k, H) or topology == "full":
        Xg = sim.X.cpu().numpy()
        assert all(np.array_equal(Xg[0], Xg[i]) for i in range(n)), "rows differ after a global step"
        assert sim.consensus_error() <= 1e-6 * np.linalg.norm(Xg)
    sim.close()


OPTION_SETS = [
    {"unroll": 1}, {"unroll": 2}, {"unroll": 8},
    {"waves": 1}, {"waves": 2}, {"waves": 8},
    {"waves": 8, "row_split": 8}, {"row_split": 1}, {"row_split": 2}, {"row_split": 4},
    {"row_lanes": 1, "row_split": 1}, {"row_lanes": 2}, {"row_lanes": 4, "row_split": 4},
    {"xcd_swizzle": 1}, {"xcd_swizzle": 1, "waves": 2, "row_split": 2},
    {"blocks_per_cu": 1}, {"blocks_per_cu": 2, "waves": 2, "row_split": 2}, {"blocks_per_cu": 1, "xcd_swizzle": 1},
    {"waves": 8, "blocks_per_cu": 1}, {"unroll": 1, "row_split": 4}, {"unroll": 2, "row_split": 2},
]


@pytest.mark.parametrize("opts", OPTION_SETS, ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
@pytest.mark.parametrize("n,d,topology", [(64, 5000, "ring"), (64, 5000, "expo1"), (20, 333, "ring"),
                                          (24, 1300, "expo1")])
def test_every_launch_geometry_gives_the_same_answer(hx, opts, n, d, topology):
    X, Mb, G = inputs.random_state(n, d, seed=7 + n)
    for k, H in ((0, 0), (1, 0), (2, 0), (4, 0), (5, 6)):
        sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.1, momentum=0.9)
        for name, v in opts.items():
            sim.set_option(name, v)
        sim.set_state(X=X, M=Mb, G=G, k=k)
        sim.step()
        X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, k, topology=topology, H=H, lr=0.1, momentum=0.9)
        assert_close(host(sim.X), X_ref, TOL_STEP, f"X k={k}")
        assert_close(host(sim.M), M_ref, TOL_STEP, f"M k={k}")
        sim.close()


@pytest.mark.parametrize("topology,k,H", [("ring", 0, 0), ("expo1", 0, 0), ("expo1", 3, 0), ("expo1", 5, 0),
                                          ("ring", 5, 6), ("none", 1, 0)])
@pytest.mark.parametrize("opts", [{"blocks_per_cu": 1, "waves": 1, "pace_gbs": 2000, "pace_min_cycle": 2},
                                  {"blocks_per_cu": 2, "waves": 2, "pace_gbs": 8000, "unroll": 4, "row_split": 1, "pace_min_cycle": 2},
                                  {"blocks_per_cu": 1, "waves": 4, "pace_gbs": 0, "unroll": 1}],
                         ids=["paced-w1", "paced-w2-u4", "persistent-unpaced"])
def test_persistent_paced_launch_matches_oracle(hx, topology, k, H, opts):
    # wide enough that the work items exceed the resident workgroups: the grid-stride
    # loop, the shared start time and the deadline waits are all exercised
    n, d = 64, 300_004
    X, Mb, G = inputs.random_state(n, d, seed=99)
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.1, momentum=0.9)
    for name, v in opts.items():
        sim.set_option(name, v)
    X_ref, M_ref = X, Mb
    sim.set_state(X=X, M=Mb, G=G, k=k)
    for j in range(3):          # several launches in a row share one pacing state
        sim.step()
        # (the W = I step is never paced: its one-shot launch keeps a single row open per workgroup anyway; the
        # global average at this width spreads rows over lanes and wavefronts, which is not paced either: its
        # paced form is checked at full size)
        want_paced = opts["pace_gbs"] and topology != "none" and not orc.is_global_step(k + j, H)
        assert int(sim.query("step_paced")) == (1 if want_paced else 0), f"step {j}: pacing is not as asked for"
        X_ref, M_ref = orc.gossip_pga_step(X_ref, M_ref, G, k + j, topology=topology, H=H, lr=0.1, momentum=0.9)
        X_ref = X_ref.astype(np.float32).astype(np.float64)
        M_ref = M_ref.astype(np.float32).astype(np.float64)
        assert_close(host(sim.X), X_ref, TOL_STEP, f"X after step {j}")
        assert_close(host(sim.M), M_ref, TOL_STEP, f"M after step {j}")
    sim.close()


@pytest.mark.parametrize("n,d,k,momentum,opts", [
    (64, 300_004, 4, 0.9, {"cycle_kernel": 1}),                       # offset 16: cycles of 4 rows
    (64, 300_004, 5, 0.9, {"cycle_kernel": 1}),                       # offset 32: cycles of 2 rows
    (64, 300_004, 5, 0.0, {"cycle_kernel": 1, "pace_gbs": 2000}),
    (64, 300_004, 4, 0.9, {"cycle_kernel": 1, "blocks_per_cu": 1, "waves": 2, "pace_gbs": 8000}),
    (1024, 4100, 9, 0.9, {"cycle_kernel": 1}),                        # offset 512
    (1024, 4100, 8, 0.9, {"cycle_kernel": 1, "blocks_per_cu": 0}),    # offset 256, one-shot launch
    (2, 1000, 0, 0.9, {"cycle_kernel": 1}),                           # n = 2: one cycle of two rows
    (4, 1000, 0, 0.5, {"cycle_kernel": 1}),                           # offset 1 on n = 4: one cycle of four rows
    (8, 999, 2, 0.9, {"cycle_kernel": 1}),                            # ragged d: the scalar tail takes the walk
    (64, 300_004, 4, 0.9, {"cycle_kernel": 0}),                       # switched off: the walk kernel
])
def test_whole_cycle_kernel_for_short_one_peer_cycles(hx, n, d, k, momentum, opts):
    X, Mb, G = inputs.random_state(n, d, seed=500 + n + k)
    for nesterov in ((False, True) if momentum else (False,)):
        sim = hx.Simulation(n, d, topology="expo1", H=0, lr=0.1, momentum=momentum)
        if nesterov:
            sim.set_nesterov(True)
        for name, v in opts.items():
            sim.set_option(name, v)
        sim.set_state(X=X, M=Mb, G=G, k=k)
        sim.step()
        # the row-streaming kernel takes the 16-byte columns of cycles of 2, 4, 8 or 16 rows unless switched off
        assert int(sim.query("step_path")) == (2 if opts["cycle_kernel"] and d % 4 == 0 else 1)
        X_ref, M_ref = orc.gossip_pga_step(X, Mb if momentum else np.zeros_like(Mb), G, k, topology="expo1", H=0,
                                           lr=0.1, momentum=momentum, nesterov=nesterov)
        assert_close(host(sim.X), X_ref, TOL_STEP, "X")
        if momentum:
            assert_close(host(sim.M), M_ref, TOL_STEP, "M")
        sim.close()


def test_padding_columns_and_inputs_are_untouched(hx):
    n, d, ld = 8, 1001, 1008
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.9, ld=ld)
    X, Mb, G = inputs.random_state(n, d, seed=3)
    sim.set_state(X=X, M=Mb, G=G, k=0)
    for buf in sim._bufs + [sim.m, sim.g]:
        buf[:, d:] = 123.0
    x_before = sim.X.clone()
    g_before = sim.G.clone()
    sim.step()
    for buf in sim._bufs + [sim.m, sim.g]:
        assert bool((buf[:, d:] == 123.0).all())
    old = [b for b in sim._bufs if b.data_ptr() != sim.X.data_ptr()][0]
    assert torch.equal(old[:, :d], x_before) and torch.equal(sim.G, g_before)
    sim.close()


# ------------------------------------------------------------------ gradients

@pytest.mark.parametrize("n,d,ld,k,seed", [(4, 64, 64, 0, 0), (5, 1003, 1003, 7, 1), (3, 4099, 4104, 123456, 0xABCDEF0123),
                                            (64, 8192, 8192, 99, 0)])
def test_synthetic_gradient_matches_counter_rng_oracle(hx, n, d, ld, k, seed):
    var = 1e-3
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0, ld=ld)
    sim.problem_synthetic(seed, var)
    sim.set_state(k=k)
    sim.local_grad()
    G_ref = orc.synthetic_grad(seed, k, n, np.arange(d), var)
    assert_close(host(sim.G), G_ref, TOL_STEP, "G")
    sim.close()


@pytest.mark.parametrize("n,d,M,B", [(3, 10, 7, 0), (8, 1000, 100, 0), (4, 1003, 20, 6), (5, 4096, 33, 33)])
def test_least_squares_gradient_and_loss(hx, n, d, M, B):
    A, b, _ = inputs.lsq_problem(n, d, M, seed=5)
    X = inputs.random_state(n, d, seed=11)[0]
    idx = inputs.batch_indices(1, n, B, M, seed=2)[0] if B else None
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
    sim.problem_lsq(A, b)
    sim.set_state(X=X)
    idx_d = sim.upload_batches(idx) if B else None
    sim.local_grad(idx_d)
    assert_close(host(sim.G), orc.lsq_grad(A, b, X, idx), TOL_STEP, "G")
    assert_close(host(sim.local_loss(idx_d)), orc.lsq_loss(A, b, X, idx), TOL_STEP, "loss")
    sim.close()


@pytest.mark.parametrize("n,d,M,B,scale", [(3, 10, 7, 0, 1.0), (32, 10000, 50, 32, 0.01), (4, 1003, 20, 6, 0.3),
                                           (4, 1003, 20, 6, 30.0), (5, 4096, 33, 16, 1.0)])
def test_logistic_gradient_and_loss(hx, n, d, M, B, scale):
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=5)
    X = inputs.random_state(n, d, seed=12, scale=scale)[0]
    idx = inputs.batch_indices(1, n, B, M, seed=2)[0] if B else None
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
    sim.problem_logreg(feat, y)
    sim.set_state(X=X)
    idx_d = sim.upload_batches(idx) if B else None
    sim.local_grad(idx_d)
    assert_close(host(sim.G), orc.logreg_grad(feat, y, X, idx), TOL_STEP, "G")
    assert_close(host(sim.local_loss(idx_d)), orc.logreg_loss(feat, y, X, idx), TOL_STEP, "loss")
    sim.close()


@pytest.mark.parametrize("n,d,M,B,seed", [(3, 40, 6, 4, 3), (6, 4099, 50, 16, 0), (4, 20000, 500, 16, 77)])
def test_virtual_feature_logistic_gradient(hx, n, d, M, B, seed):
    mu_var = 0.5
    y = inputs.virtual_labels(n, M, seed)
    X = inputs.random_state(n, d, seed=13, scale=1.0 / math.sqrt(d))[0]
    idx = inputs.batch_indices(1, n, B, M, seed=4)[0]
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
    sim.problem_logreg_virtual(seed, y, mu_var)
    sim.set_state(X=X)
    idx_d = sim.upload_batches(idx)
    sim.local_grad(idx_d)
    assert_close(host(sim.G), orc.logreg_virtual_grad(seed, y, X, idx, mu_var), TOL_STEP, "G")
    sim.close()


# ------------------------------------------------------------------ reductions

@pytest.mark.parametrize("n,d,pad", [(1, 5, 0), (8, 1000, 0), (64, 4099, 1), (1024, 777, 0)])
def test_mean_and_consensus_error(hx, n, d, pad):
    base = inputs.initial_point(d, seed=1).astype(np.float64) * 100.0
    dev = inputs.random_state(n, d, seed=21, scale=1e-3)[0].astype(np.float64)
    X = (base[None, :] + dev).astype(np.float32)          # small spread on a large common part
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0, ld=d + pad)
    sim.set_state(X=X)
    assert_close(host(sim.mean()), orc.node_mean(X), TOL_STEP, "mean")
    ce, ce_ref = sim.consensus_error(), orc.consensus_error(X)
    assert abs(ce - ce_ref) <= TOL_STEP * ce_ref + 1e-30
    sim.close()


# ------------------------------------------------------------------ whole trajectories

def _run_pair(sim, ref, T, grad_gpu, grad_ref, lockstep_every=1):
    """Free-running GPU and oracle trajectories plus a lock-step check: at every
    step the oracle is also advanced once from the GPU's own state."""
    worst_lock = 0.0
    for k in range(T):
        grad_gpu(k)
        if k % lockstep_every == 0:
            Xg, Gg = host(sim.X), host(sim.G)
            Mg = host(sim.M) if sim.M is not None else np.zeros_like(Xg)
            assert_close(Gg, grad_ref(k, Xg), TOL_STEP, f"G at step {k}")
            X1, _ = orc.gossip_pga_step(Xg, Mg, Gg, k, topology=ref.topology, H=ref.H, lr=ref.lr,
                                        momentum=ref.momentum)
        sim.step()
        if k % lockstep_every == 0:
            emax, efro = rel_errors(host(sim.X), X1)
            worst_lock = max(worst_lock, emax, efro)
            assert emax <= TOL_STEP and efro <= TOL_STEP, f"lock-step X at step {k}: {emax:.2e} {efro:.2e}"
        ref.step(grad_ref(k, ref.X))
    return worst_lock


def test_cfg1_least_squares_ring_full_trajectory(hx):
    c = inputs.CONFIGS["cfg1"]
    n, d, M, T = c["n"], c["d"], c["M"], c["T"]
    A, b, _ = inputs.lsq_problem(n, d, M, c["seed"], c["noise_std"])
    sim = hx.Simulation(n, d, topology="ring", H=c["H"], lr=c["lr"], momentum=c["momentum"])
    sim.problem_lsq(A, b)
    ref = orc.GossipPGA(n, d, topology="ring", H=c["H"], lr=c["lr"], momentum=c["momentum"], storage="f32")
    worst = _run_pair(sim, ref, T, lambda k: sim.local_grad(), lambda k, X: orc.lsq_grad(A, b, X))
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    Xg = sim.X.cpu().numpy()
    assert all(np.array_equal(Xg[0], Xg[i]) for i in range(n))     # step 199 is a global average
    # the decentralised run has made progress on the global objective
    f0 = orc.lsq_loss(A, b, np.zeros((n, d))).mean()
    f1 = orc.lsq_loss(A, b, host(sim.X)).mean()
    assert f1 < 0.1 * f0
    print(f"cfg1: worst lock-step error {worst:.2e}, final {rel_errors(host(sim.X), ref.X)}")
    sim.close()


def test_cfg2_logistic_one_peer_trajectory(hx):
    c = inputs.CONFIGS["cfg2"]
    n, d, M, B, T = c["n"], c["d"], c["M"], c["B"], c["T"]
    feat, y, _ = inputs.logreg_problem(n, d, M, c["seed"], c["mu_var"], c["label_noise_std"])
    idx = inputs.batch_indices(T, n, B, M, c["seed"])
    sim = hx.Simulation(n, d, topology="expo1", H=c["H"], lr=c["lr"], momentum=c["momentum"])
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(idx)
    kw = dict(topology="expo1", H=c["H"], lr=c["lr"], momentum=c["momentum"])
    ref = orc.GossipPGA(n, d, storage="f32", **kw)
    ref64 = orc.GossipPGA(n, d, storage="f64", **kw)
    # Every step is checked in lock-step (oracle advanced once from the GPU's state).
    # The free-running comparison is meaningful only while the problem itself does not
    # amplify rounding: this recipe (un-normalised 10^4-dimensional features, lr 0.05) is
    # chaotic, which the oracle shows on its own (fp32-stored vs all-fp64 trajectories).
    T_free = 16
    free_err = None
    for k in range(T):
        sim.local_grad(idx_d[k])
        Xg, Gg, Mg = host(sim.X), host(sim.G), host(sim.M)
        assert_close(Gg, orc.logreg_grad(feat, y, Xg, idx[k]), TOL_STEP, f"G at step {k}")
        X1, M1 = orc.gossip_pga_step(Xg, Mg, Gg, k, **kw)
        sim.step()
        assert_close(host(sim.X), X1, TOL_STEP, f"lock-step X at step {k}")
        assert_close(host(sim.M), M1, TOL_STEP, f"lock-step M at step {k}")
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]))
        ref64.step(orc.logreg_grad(feat, y, ref64.X, idx[k]))
        if k + 1 == T_free:
            free_err = max(rel_errors(host(sim.X), ref.X))
            floor = max(rel_errors(ref.X, ref64.X))
            assert free_err <= TOL_FINAL, f"free-running error after {T_free} steps {free_err:.2e} (oracle floor {floor:.2e})"
    gpu_vs_ref = max(rel_errors(host(sim.X), ref.X))
    floor = max(rel_errors(ref.X, ref64.X))
    print(f"cfg2: free-running T={T}: GPU vs oracle {gpu_vs_ref:.3e}; oracle fp32-storage vs fp64 {floor:.3e}; "
          f"after {T_free} steps {free_err:.3e}")
    # the GPU trajectory is no further from the oracle than the oracle is from itself
    assert gpu_vs_ref <= max(TOL_FINAL, 3.0 * floor)
    sim.close()


def test_cfg2_shapes_with_normalised_features_free_running(hx):
    # Same shapes, graph, period, momentum and T as cfg2, with features scaled by
    # 1/sqrt(d) so that the iteration is contractive: here the free-running final
    # iterates can be held to TOL_FINAL.
    c = inputs.CONFIGS["cfg2"]
    n, d, M, B, T = c["n"], c["d"], 200, c["B"], c["T"]
    feat, y, _ = inputs.logreg_problem(n, d, M, c["seed"] + 1, c["mu_var"], c["label_noise_std"])
    feat = (feat / math.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, B, M, c["seed"] + 1)
    sim = hx.Simulation(n, d, topology="expo1", H=c["H"], lr=c["lr"], momentum=c["momentum"])
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(idx)
    ref = orc.GossipPGA(n, d, topology="expo1", H=c["H"], lr=c["lr"], momentum=c["momentum"], storage="f32")
    for k in range(T):
        sim.local_grad(idx_d[k])
        sim.step()
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]))
        if k % 50 == 49:
            assert_close(host(sim.X), ref.X, TOL_FINAL, f"free-running X at step {k}")
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    assert_close(host(sim.M), ref.M, TOL_FINAL, "final momentum")
    sim.close()


def _work_item_slabs(d, width=1024, resident=1024):
    """Column slabs that sit on particular work items of the persistent launches: with 4
    wavefronts of 64 lanes x 4 columns a tile group is 1024 columns, and a launch of
    `resident` workgroups gives workgroup b the tile groups b, b + resident, ...  Returned:
    the first and last tile group of the first, second and last workgroup, the tile groups
    on either side of the first wrap-around, and the ragged end of the array."""
    groups = (d + width - 1) // width
    last_round = ((groups - 1) // resident) * resident
    picks = {0, 1, resident - 1, resident, resident + 1, 2 * resident - 1, groups - 1, groups - 2,
             last_round, last_round + 1, last_round - 1, groups // 2}
    starts = sorted(min(max(g, 0), groups - 1) * width for g in picks)
    cols = np.concatenate([np.arange(s0, min(d, s0 + width)) for s0 in starts])
    return np.unique(cols)


def _slab_trajectory(hx, cfg_name, topology, n_slabs, width, T=None, opts=None, nesterov=False, H=None, gossip_path=None):
    """Column-separable workloads (synthetic gradients): the GPU runs the full array, the
    oracle follows column slabs (evenly spaced ones plus slabs placed on the first and last
    tile groups of several work items of the persistent launch).  Every step is checked in
    lock-step at TOL_STEP - the oracle advanced once from the GPU's own X, M, G on the slab
    columns - and G against the counter RNG; the free-running oracle trajectory is held to
    TOL_FINAL at every step and for the final iterates."""
    c = inputs.CONFIGS[cfg_name]
    n, d = c["n"], c["d"]
    T = c["T"] if T is None else T
    c = dict(c, H=c["H"] if H is None else H)
    cols = np.union1d(inputs.slab_columns(d, n_slabs, width), _work_item_slabs(d))
    sim = hx.Simulation(n, d, topology=topology, H=c["H"], lr=c["lr"], momentum=c["momentum"])
    if nesterov:
        sim.set_nesterov(True)
    for name, v in (opts or {}).items():
        sim.set_option(name, v)
    sim.problem_synthetic(c["seed"], c["grad_var"])
    cols_d = torch.as_tensor(cols, device=sim.device)
    kw = dict(topology=topology, H=c["H"], lr=c["lr"], momentum=c["momentum"], nesterov=nesterov)
    ref = orc.GossipPGA(n, len(cols), storage="f32", **kw)
    slab = lambda t: host(t.index_select(1, cols_d))
    worst = worst_lock = 0.0
    for k in range(T):
        sim.local_grad()
        G_ref = orc.synthetic_grad(c["seed"], k, n, cols, c["grad_var"])
        Xs, Ms, Gs = slab(sim.X), slab(sim.M), slab(sim.G)
        assert_close(Gs, G_ref, TOL_STEP, f"G at step {k}")
        X1, M1 = orc.gossip_pga_step(Xs, Ms, Gs, k, **kw)
        sim.step()
        if gossip_path is not None and not orc.is_global_step(k, H if H is not None else c["H"]):
            assert int(sim.query("step_path")) in gossip_path, f"step {k} ran as path {int(sim.query('step_path'))}"
        ref.step(G_ref)
        Xn = slab(sim.X)
        for got, want, what in ((Xn, X1, "X"), (slab(sim.M), M1, "M")):
            emax, efro = rel_errors(got, want)
            worst_lock = max(worst_lock, emax, efro)
            assert emax <= TOL_STEP and efro <= TOL_STEP, \
                f"{cfg_name}/{topology} lock-step {what} at step {k}: {emax:.2e} {efro:.2e}"
        emax, efro = rel_errors(Xn, ref.X)
        worst = max(worst, emax, efro)
        assert emax <= TOL_FINAL and efro <= TOL_FINAL, f"{cfg_name}/{topology} free-running step {k}: {emax:.2e} {efro:.2e}"
        if orc.is_global_step(k, c["H"]):     # rows identical: error far below the iterate's own norm
            assert sim.consensus_error() <= 1e-6 * np.linalg.norm(ref.X) * math.sqrt(d / len(cols))
    assert_close(slab(sim.X), ref.X, TOL_FINAL, "final iterate")
    assert_close(slab(sim.M), ref.M, TOL_FINAL, "final momentum")
    ce = sim.consensus_error()
    ce_slab = orc.consensus_error(ref.X)
    # slab columns are a sample of iid columns: consensus error scales with sqrt(d / |slab|)
    assert ce == pytest.approx(ce_slab * math.sqrt(d / len(cols)), rel=0.05)
    print(f"{cfg_name}/{topology}: {T} steps, {len(cols)} slab columns, worst lock-step error {worst_lock:.2e}, "
          f"worst free-running error {worst:.2e}")
    sim.close()
    del sim
    torch.cuda.empty_cache()


@pytest.mark.parametrize("topology", ["ring", "expo1"])
def test_cfg3_resnet50_sized_slabs(hx, topology):
    _slab_trajectory(hx, "cfg3", topology, n_slabs=32, width=1024, gossip_path=(1, 2))    # stencil walk / row-streaming kernel


@pytest.mark.parametrize("topology,nesterov", [("grid", False), ("expo", True), ("ring", True)])
def test_cfg3_sized_slabs_sparse_W_and_nesterov(hx, topology, nesterov):
    # the widened variants at the benchmark's full size: LDS-tile kernel (grid, static exponential
    # graph) and Nesterov momentum, two averaging periods
    _slab_trajectory(hx, "cfg3", topology, n_slabs=32, width=1024, T=17, nesterov=nesterov, H=8,
                     gossip_path=(1,) if topology == "ring" else (4,))


@pytest.mark.parametrize("topology,path", [("grid", 5), ("expo", 6)])
def test_cfg5_sized_slabs_sparse_W(hx, topology, path):
    # n = 1024 rows (synthetic gradients on the cfg5 shape so that the oracle can follow column slabs): the
    # 32 x 32 grid is banded and takes the sliding-window kernel, the static exponential graph the two passes
    # (local update written over the old iterate, then the sparse product)
    c = dict(inputs.CONFIGS["cfg5"], problem="synthetic", grad_var=1e-3)
    inputs.CONFIGS["cfg5_synth"] = c
    try:
        _slab_trajectory(hx, "cfg5_synth", topology, n_slabs=16, width=256, T=10, H=8, gossip_path=(path,))
    finally:
        del inputs.CONFIGS["cfg5_synth"]


def test_cfg4_bert_base_sized_slabs(hx):
    _slab_trajectory(hx, "cfg4", "expo1", n_slabs=32, width=1024, gossip_path=(1, 2))


_REPLICA = {}


def _cfg5_replica_data():
    """n = 1024 nodes as in cfg5 with d and M reduced so that the oracle can run the
    whole (non-separable) logistic trajectory: features are materialised once from the
    oracle's own counter RNG."""
    if not _REPLICA:
        c = inputs.CONFIGS["cfg5"]
        n, d, M, B, T = c["n"], 2048, 64, c["B"], 40
        y = inputs.virtual_labels(n, M, c["seed"])
        idx = inputs.batch_indices(T, n, B, M, c["seed"])
        feat = np.stack([orc.virtual_features(c["seed"], i, np.arange(M), np.arange(d), c["mu_var"]).astype(np.float32)
                         for i in range(n)])
        _REPLICA.update(n=n, d=d, M=M, B=B, T=T, y=y, idx=idx, feat=feat)
    return _REPLICA


@pytest.mark.parametrize("topology", ["ring", "expo1"])
@pytest.mark.parametrize("H", [1, 8, 64, 0])
def test_cfg5_reduced_width_replica(hx, topology, H):
    c = inputs.CONFIGS["cfg5"]
    r = _cfg5_replica_data()
    n, d, T, y, idx, feat = r["n"], r["d"], r["T"], r["y"], r["idx"], r["feat"]
    lr = c["lr"] / 8.0    # keeps this reduced problem in the contractive regime
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=lr, momentum=c["momentum"])
    sim.problem_logreg_virtual(c["seed"], y, c["mu_var"])
    idx_d = sim.upload_batches(idx)
    ref = orc.GossipPGA(n, d, topology=topology, H=H, lr=lr, momentum=c["momentum"], storage="f32")
    for k in range(T):
        sim.local_grad(idx_d[k])
        sim.step()
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]))
        ce, ce_ref = sim.consensus_error(), orc.consensus_error(ref.X)
        if H == 1 or orc.is_global_step(k, H):
            assert ce <= 1e-6 * np.linalg.norm(ref.X) + 1e-30
        else:
            assert ce == pytest.approx(ce_ref, rel=1e-3)
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    sim.close()


# ------------------------------------------------------------------ error paths (host-side, no kernel runs)

def test_error_paths_return_status_codes(hx):
    from paper_2105_09080_amd import binding as B
    with pytest.raises(B.GpgaError) as e:
        B.gpga_create(0, 10, "ring", 1, 0.1, 0.0)
    assert e.value.status == B.GPGA_EINVAL
    for bad in (dict(d=0), dict(H=-1), dict(lr=float("nan")), dict(momentum=1.0), dict(topology=9)):
        kw = dict(n=4, d=8, topology="ring", H=1, lr=0.1, momentum=0.0)
        kw.update(bad)
        with pytest.raises(B.GpgaError):
            B.gpga_create(kw["n"], kw["d"], kw["topology"], kw["H"], kw["lr"], kw["momentum"])
    ctx = B.gpga_create(4, 8, "ring", 1, 0.1, 0.9)
    with pytest.raises(B.GpgaError) as e:
        B.gpga_step(ctx)
    assert e.value.status == B.GPGA_ESTATE and "bound" in str(e.value)
    t = torch.zeros((4, 8), device="cuda")
    t2 = torch.zeros((4, 8), device="cuda")
    with pytest.raises(B.GpgaError) as e:
        B.gpga_bind(ctx, t, t, t2, t2, 8)          # x_new aliases x
    assert e.value.status == B.GPGA_EINVAL
    m0, g0 = torch.zeros((4, 8), device="cuda"), torch.zeros((4, 8), device="cuda")
    big = torch.zeros(4 * 8 + 16, device="cuda")
    for args in ((t, t2, g0, g0), (t, t2, t, g0), (t, t2, m0, t2), (big[:32], big[16:48], m0, g0)):
        with pytest.raises(B.GpgaError) as e:       # any two of the four arrays overlapping
            B.gpga_bind(ctx, *args, 8)
        assert e.value.status == B.GPGA_EINVAL and "overlap" in str(e.value)
    with pytest.raises(B.GpgaError):
        B.gpga_bind(ctx, t, t2, None, t2, 8)       # momentum != 0 needs m
    with pytest.raises(B.GpgaError):
        B.gpga_bind(ctx, t, t2, m0, g0, 4)         # ld < d
    m, g = torch.zeros((4, 8), device="cuda"), torch.zeros((4, 8), device="cuda")
    B.gpga_bind(ctx, t, t2, m, g, 8)
    with pytest.raises(B.GpgaError) as e:
        B.gpga_local_grad(ctx, None, 0)            # no problem attached
    assert e.value.status == B.GPGA_ESTATE
    with pytest.raises(B.GpgaError):
        B.gpga_set_option(ctx, "unroll", 3)
    with pytest.raises(B.GpgaError):
        B.gpga_set_option(ctx, "nonsense", 1)
    B.gpga_destroy(ctx)


# ------------------------------------------------------------------ adaptive period (Algorithm 2)

@pytest.mark.parametrize("topology", ["ring", "expo1"])
def test_gossip_aga_trajectory_and_period_sequence(hx, topology):
    n, d, M, B, T = 16, 512, 64, 8, 80
    H_init, K_w, H_max, lr, mu = 2, 8, 12, 0.5, 0.9
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=21)
    feat = (feat / math.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, B, M, seed=21)
    sim = hx.Simulation(n, d, topology=topology, H=0, lr=lr, momentum=mu)
    sim.problem_logreg(feat, y)
    sim.aga_enable(H_init, K_w, H_max)
    idx_d = sim.upload_batches(idx)
    ref = orc.GossipAGA(n, d, topology=topology, H_init=H_init, warmup_iters=K_w, H_max=H_max, lr=lr,
                        momentum=mu, storage="f32")
    periods = []
    for k in range(T):
        loss = sim.local_loss(idx_d[k])
        sim.local_grad(idx_d[k])
        sim.aga_step(loss)
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]), orc.logreg_loss(feat, y, ref.X, idx[k]))
        periods.append(sim.period)
        assert sim.period == ref.H, f"period differs at step {k}: {sim.period} vs {ref.H}"
        if ref.history and ref.history[-1][0] == k:          # a global average just happened
            Xg = sim.X.cpu().numpy()
            assert all(np.array_equal(Xg[0], Xg[i]) for i in range(n))
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    assert_close(host(sim.M), ref.M, TOL_FINAL, "final momentum")
    assert len(set(periods)) > 1, "the period never adapted in this run"
    with pytest.raises(Exception):
        sim.step()                                            # plain step is refused while AGA is on
    sim.close()


def test_out_of_range_sample_indices_poison_only_their_node_and_touch_nothing(hx):
    # indices outside [0, M) are checked by the kernels: never used as an address, the node's
    # gradient row and loss become NaN, every other node is computed as usual
    n, d, M, B = 4, 1003, 20, 6
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=9)
    idx = inputs.batch_indices(1, n, B, M, seed=9)[0].copy()
    bad = idx.copy()
    bad[1, 2] = M              # one past the end
    bad[3, 0] = -1
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(np.stack([idx, bad]))
    X = inputs.random_state(n, d, seed=9)[0]
    sim.set_state(X=X)
    sim.local_grad(idx_d[1])
    G_bad = host(sim.G)
    loss_bad = host(sim.local_loss(idx_d[1]))
    G_ref = orc.logreg_grad(feat, y, X.astype(np.float64), idx)
    assert np.isnan(G_bad[1]).all() and np.isnan(G_bad[3]).all()
    assert np.isnan(loss_bad[[1, 3]]).all() and np.isfinite(loss_bad[[0, 2]]).all()
    assert_close(G_bad[[0, 2]], G_ref[[0, 2]], TOL_STEP, "untouched nodes")
    sim.close()
    # the virtual-feature problem reads labels through the same indices
    yv = inputs.virtual_labels(n, M, seed=9)
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
    sim.problem_logreg_virtual(9, yv, 0.5)
    idx_d = sim.upload_batches(np.stack([idx, bad]))
    sim.set_state(X=X)
    sim.local_grad(idx_d[1])
    G_bad = host(sim.G)
    assert np.isnan(G_bad[1]).all() and np.isnan(G_bad[3]).all() and np.isfinite(G_bad[[0, 2]]).all()
    sim.close()
