"""GPU parity of the optimizer variants behind the C ABI: Nesterov momentum in
the fused step (gossip and global-average kernels) and the step-size schedules,
compared with the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import gpga_oracle as orc
from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_STEP = 1e-5      # one call on identical inputs
TOL_FINAL = 1e-4     # final iterates of a free-running trajectory


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


NESTEROV_CASES = [
    # n, d, ld_pad, topology, momentum, H, k
    (1, 5, 0, "ring", 0.9, 0, 0),
    (3, 256, 0, "ring", 0.5, 0, 1),
    (8, 1031, 1, "ring", 0.9, 0, 5),          # vector path plus 3-column tail
    (8, 1030, 2, "ring", 0.9, 0, 5),          # scalar path
    (64, 4100, 0, "ring", 0.9, 48, 47),       # global average
    (6, 300, 0, "expo1", 0.9, 0, 2),
    (32, 10000, 0, "expo1", 0.9, 16, 4),
    (32, 10000, 0, "expo1", 0.9, 16, 15),     # global average
    (1024, 520, 0, "ring", 0.9, 8, 7),        # global average, rows split over lanes and waves
    (1024, 520, 0, "expo1", 0.9, 0, 3),
    (16, 777, 0, "none", 0.9, 5, 1),
    (16, 777, 0, "full", 0.3, 0, 1),
    (64, 300_004, 0, "ring", 0.9, 0, 0),      # wide rows: several column tiles per workgroup
    (64, 300_004, 0, "expo1", 0.9, 6, 5),     # ... and the global average on them
]


@pytest.mark.parametrize("n,d,pad,topology,momentum,H,k", NESTEROV_CASES)
def test_nesterov_step_matches_oracle(hx, n, d, pad, topology, momentum, H, k):
    X, Mb, G = inputs.random_state(n, d, seed=4000 + n + d + k)
    lr = 0.37
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=lr, momentum=momentum, ld=d + pad)
    sim.set_nesterov(True)
    sim.set_state(X=X, M=Mb, G=G, k=k)
    sim.step()
    X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, k, topology=topology, H=H, lr=lr, momentum=momentum,
                                       nesterov=True)
    X_hb, _ = orc.gossip_pga_step(X, Mb, G, k, topology=topology, H=H, lr=lr, momentum=momentum)
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    assert rel_errors(host(sim.X), X_hb)[0] > 1e-3       # and it is not the heavy-ball result
    if orc.is_global_step(k, H) or topology == "full":
        Xg = sim.X.cpu().numpy()
        assert all(np.array_equal(Xg[0], Xg[i]) for i in range(n))
    sim.close()


@pytest.mark.parametrize("topology,k,path", [("ring", 0, 1), ("expo1", 0, 1), ("expo1", 4, 2)])
def test_nesterov_step_in_paced_persistent_launches(hx, topology, k, path):
    # the Nesterov variants of the walk and of the row-streaming kernel as paced persistent launches
    # (forced by options at a size the oracle handles whole; the default launches of large problems are
    # checked at full size)
    n, d = 64, 300_004
    X, Mb, G = inputs.random_state(n, d, seed=4100 + k)
    sim = hx.Simulation(n, d, topology=topology, H=0, lr=0.37, momentum=0.9)
    sim.set_nesterov(True)
    opts = {"blocks_per_cu": 2, "pace_gbs": 5000, "cycle_kernel": 1}
    if path == 1:
        opts["row_split"] = 1          # one walker per cycle (the row-streaming kernel never splits rows)
    for name, v in opts.items():
        sim.set_option(name, v)
    sim.set_state(X=X, M=Mb, G=G, k=k)
    sim.step()
    assert (int(sim.query("step_path")), int(sim.query("step_paced"))) == (path, 1)
    X_ref, M_ref = orc.gossip_pga_step(X, Mb, G, k, topology=topology, H=0, lr=0.37, momentum=0.9, nesterov=True)
    assert_close(host(sim.X), X_ref, TOL_STEP, "X")
    assert_close(host(sim.M), M_ref, TOL_STEP, "M")
    sim.close()


def test_nesterov_needs_momentum_and_can_be_switched_off(hx):
    from paper_2105_09080_amd import binding as B
    sim = hx.Simulation(4, 64, topology="ring", H=0, lr=0.1, momentum=0.0)
    with pytest.raises(B.GpgaError) as e:
        sim.set_nesterov(True)
    assert e.value.status == B.GPGA_EINVAL
    sim.close()
    n, d = 8, 515
    X, Mb, G = inputs.random_state(n, d, seed=5)
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.9)
    sim.set_nesterov(True)
    sim.set_nesterov(False)
    sim.set_state(X=X, M=Mb, G=G, k=0)
    sim.step()
    X_ref, _ = orc.gossip_pga_step(X, Mb, G, 0, topology="ring", H=0, lr=0.1, momentum=0.9)
    assert_close(host(sim.X), X_ref, TOL_STEP, "heavy-ball again")
    sim.close()


def _f32(v):
    return float(np.float32(v))


def _ulp_close(a, b):
    a32, b32 = np.float32(a), np.float32(b)
    return a32 == b32 or abs(float(a32) - float(b32)) <= float(np.spacing(np.float32(max(abs(a32), abs(b32)))))


def test_schedules_give_the_oracles_step_size_at_every_iteration(hx):
    from paper_2105_09080_amd import binding as B
    sim = hx.Simulation(4, 16, topology="ring", H=0, lr=0.5, momentum=0.0)
    ctx = sim.ctx
    assert B.gpga_lr(ctx) == _f32(0.5)

    base = _f32(0.2)
    B.gpga_lr_schedule_step(ctx, base, 1000, 0.5)
    for k in (0, 1, 999, 1000, 1999, 2000, 7500, 40_000, 200_000):
        B.gpga_set_iter(ctx, k)
        assert _ulp_close(B.gpga_lr(ctx), orc.lr_step_decay(k, base, 1000, 0.5)), k

    ipe = 1281167 // 8192
    base, start, fac = _f32(3.2), _f32(0.1), _f32(0.1)
    ms = [30 * ipe, 60 * ipe, 90 * ipe]
    B.gpga_lr_schedule_milestones(ctx, base, 5 * ipe, start, ms, fac)
    for k in [0, 1, 17, 5 * ipe - 1, 5 * ipe, 30 * ipe - 1, 30 * ipe, 60 * ipe, 90 * ipe - 1, 90 * ipe, 120 * ipe]:
        B.gpga_set_iter(ctx, k)
        assert _ulp_close(B.gpga_lr(ctx), orc.lr_warmup_milestones(k, base, 5 * ipe, start, ms, fac)), k

    base, T, Kw, power = _f32(3.75e-4), 112608, 2000, _f32(0.5)
    B.gpga_lr_schedule_poly(ctx, base, Kw, T, power)
    for k in [0, 1, Kw - 1, Kw, Kw + 1, 50_000, T - 1, T, T + 10]:
        B.gpga_set_iter(ctx, k)
        assert _ulp_close(B.gpga_lr(ctx), orc.lr_poly(k, base, Kw, T, power)), k

    B.gpga_set_lr(ctx, 0.25)                      # a constant detaches the schedule
    B.gpga_set_iter(ctx, 12345)
    assert B.gpga_lr(ctx) == 0.25

    bad = [lambda: B.gpga_lr_schedule_step(ctx, 0.1, 0, 0.5),
           lambda: B.gpga_lr_schedule_step(ctx, float("nan"), 10, 0.5),
           lambda: B.gpga_lr_schedule_milestones(ctx, 0.1, -1, 0.0, [5], 0.1),
           lambda: B.gpga_lr_schedule_milestones(ctx, 0.1, 0, 0.0, list(range(17)), 0.1),
           lambda: B.gpga_lr_schedule_milestones(ctx, 0.1, 0, 0.0, [-4], 0.1),
           lambda: B.gpga_lr_schedule_poly(ctx, 0.1, 10, 10, 1.0),
           lambda: B.gpga_lr_schedule_poly(ctx, 0.1, 0, 10, 0.0)]
    for f in bad:
        with pytest.raises(B.GpgaError) as e:
            f()
        assert e.value.status == B.GPGA_EINVAL
    assert B.gpga_lr(ctx) == 0.25                 # rejected calls change nothing
    sim.close()


@pytest.mark.parametrize("topology,nesterov", [("ring", False), ("expo1", True)])
def test_trajectory_with_halving_schedule_and_nesterov(hx, topology, nesterov):
    # logistic regression in the shape family of the paper's simulation (Sec. 5.1), scaled
    # features so that the trajectory is contractive; gamma = 0.2 halved every 40 iterations
    n, d, M, Bsz, T, H = 20, 1003, 60, 8, 200, 16
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=3, mu_var=0.5, label_noise_std=0.1)
    feat = (feat / np.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, Bsz, M, seed=3)
    base = _f32(0.2)
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=base, momentum=0.9)
    sim.set_nesterov(nesterov)
    from paper_2105_09080_amd import binding as B
    B.gpga_lr_schedule_step(sim.ctx, base, 40, 0.5)
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(idx)
    ref = orc.GossipPGA(n, d, topology=topology, H=H, lr=lambda k: orc.lr_step_decay(k, base, 40, 0.5),
                        momentum=0.9, nesterov=nesterov, storage="f32")
    for k in range(T):
        assert sim.lr == ref.lr_at(k)
        sim.local_grad(idx_d[k])
        # lock-step: one oracle step from the GPU's own state
        Xg, Gg, Mg = host(sim.X), host(sim.G), host(sim.M)
        X1, _ = orc.gossip_pga_step(Xg, Mg, Gg, k, topology=topology, H=H, lr=ref.lr_at(k), momentum=0.9,
                                    nesterov=nesterov)
        sim.step()
        assert_close(host(sim.X), X1, TOL_STEP, f"lock-step X at {k}")
        ref.step(orc.logreg_grad(feat, y, ref.X, idx[k]))
    assert_close(host(sim.X), ref.X, TOL_FINAL, "final iterate")
    assert_close(host(sim.M), ref.M, TOL_FINAL, "final momentum")
    sim.close()
