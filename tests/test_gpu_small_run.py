"""GPU parity of the single-workgroup trajectory path of gpga_run (small problems: the whole
iteration - stored-feature gradients, momentum, local update, gossip or global average,
consensus trace - inside one launch) against the CPU oracle and against the
kernel-per-stage path, through the C ABI."""
import math
import time

import numpy as np
import pytest

from oracle import gpga_oracle as orc
from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_STEP = 1e-5
TOL_FINAL = 1e-4
LR = 0.2


@pytest.fixture(scope="module")
def hx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import harness
    return harness


def rel(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300)


def make_problem(kind, n, d, M, seed):
    if kind == "logreg":
        feat, y, _ = inputs.logreg_simulation_problem(n, d, M, seed=seed)
        return feat, y, orc.logreg_grad, orc.logreg_loss
    A, b, _ = inputs.lsq_problem(n, d, M, seed=seed)
    return (A / math.sqrt(d)).astype(np.float32), b, orc.lsq_grad, orc.lsq_loss


def random_W(n, seed):
    rng = np.random.default_rng(seed)
    w = rng.random(4)
    w /= w.sum()
    W = w[0] * np.eye(n)
    for t in range(3):
        W += w[t + 1] * np.eye(n)[rng.permutation(n)]
    return W.astype(np.float32).astype(np.float64)


def build(hx, kind, n, d, M, topology, H, momentum, nesterov, seed, small):
    feat, tgt, grad, _ = make_problem(kind, n, d, M, seed)
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=LR, momentum=momentum)
    W = None
    if topology == "custom":
        W = random_W(n, seed)
        sim.set_mixing(W)
    if nesterov:
        sim.set_nesterov(True)
    sim.set_option("small_run", 1 if small else 0)
    (sim.problem_logreg if kind == "logreg" else sim.problem_lsq)(feat, tgt)
    return sim, feat, tgt, grad, W


CASES = [
    # kind, n, d, M, B, topology, H, momentum, nesterov, T, k0
    ("logreg", 20, 10, 400, 1, "ring", 16, 0.0, False, 60, 0),          # the shape of the Sec. 5.1 simulation
    ("logreg", 50, 10, 200, 1, "ring", 16, 0.0, False, 40, 0),
    ("logreg", 100, 10, 100, 1, "grid", 16, 0.0, False, 40, 0),
    ("logreg", 100, 10, 100, 1, "expo", 0, 0.0, False, 30, 5),
    ("logreg", 20, 10, 300, 4, "expo1", 6, 0.9, False, 50, 3),
    ("logreg", 20, 10, 300, 4, "expo1", 6, 0.9, True, 50, 3),
    ("logreg", 7, 33, 50, 5, "ring", 3, 0.5, False, 25, 0),             # d not a multiple of 4, prime n
    ("logreg", 12, 10, 80, 2, "custom", 5, 0.9, True, 30, 0),
    ("logreg", 16, 10, 80, 2, "full", 0, 0.9, False, 20, 0),            # W = J: average every iteration
    ("logreg", 16, 10, 80, 2, "none", 4, 0.0, False, 20, 0),            # Local SGD
    ("logreg", 1, 10, 80, 3, "ring", 2, 0.9, False, 10, 0),
    ("logreg", 2, 5, 40, 1, "ring", 0, 0.0, False, 12, 0),
    ("lsq", 8, 100, 40, 8, "ring", 4, 0.0, False, 40, 0),
    ("lsq", 8, 64, 20, 0, "expo1", 4, 0.9, False, 30, 1),               # full batch
    ("logreg", 64, 128, 30, 2, "grid", 8, 0.9, False, 20, 0),           # n d = 8192: the largest state taken
    ("lsq", 2, 100, 30, 4, "ring", 3, 0.9, False, 15, 0),               # long rows, a single pass of lane groups
    ("logreg", 10, 24, 60, 3, "expo1", 4, 0.9, False, 20, 0),           # groups of 32 lanes
    ("logreg", 100, 10, 50, 4, "ring", 16, 0.0, False, 20, 0),          # 400 (node, sample) pairs: seven passes
    ("logreg", 20, 10, 100, 1, "ring", 16, 0.0, False, 301, 0),         # two launches (256 + 45 iterations), the second odd
]


@pytest.mark.parametrize("kind,n,d,M,B,topology,H,momentum,nesterov,T,k0", CASES)
def test_trajectory_matches_the_oracle_driver(hx, kind, n, d, M, B, topology, H, momentum, nesterov, T, k0):
    from paper_2105_09080_amd import binding as Bn
    seed = 31 * n + d + T
    sim, feat, tgt, grad, W = build(hx, kind, n, d, M, topology, H, momentum, nesterov, seed, small=True)
    idx = inputs.batch_indices(T, n, B, M, seed=seed) if B else None
    x0 = inputs.initial_point(d, seed=seed).astype(np.float32) * 0.1
    sim.set_state(X=np.tile(x0, (n, 1)), M=np.zeros((n, d), np.float32), k=k0)
    trace = sim.attach_trace(k0 + T)
    bufs = [b.data_ptr() for b in sim._bufs]
    x_before = sim.X.data_ptr()
    sim.run(T, sim.upload_batches(idx) if B else None)
    assert int(sim.query("step_path")) == 7, "gpga_run did not take the single-workgroup path on this problem"
    # the live X sits where T separate steps would leave it: the roles of x / x_new swap once per iteration
    assert sim.k == k0 + T and sim.X.data_ptr() == bufs[(bufs.index(x_before) + T) % 2]
    ref = orc.GossipPGA(n, d, topology=topology, H=H, lr=LR, momentum=momentum, nesterov=nesterov, x0=x0,
                        storage="f32", W=W)
    ref.k = k0
    consensus, G_last = [], None
    for j in range(T):
        G_last = grad(feat, tgt, ref.X, None if idx is None else idx[j])
        ref.step(G_last)
        consensus.append(orc.consensus_error(ref.X))
    assert rel(sim.X.cpu().numpy(), ref.X) <= TOL_FINAL
    if momentum:
        assert rel(sim.M.cpu().numpy(), ref.M) <= TOL_FINAL
    assert rel(sim.G.cpu().numpy(), G_last) <= TOL_FINAL               # g holds the last iteration's gradients
    got = trace.cpu().numpy()[k0:k0 + T]
    assert np.abs(got - np.array(consensus)).max() <= TOL_FINAL * (np.linalg.norm(ref.X) + 1e-30)
    for j in range(T):                                                 # exactly zero right after an average
        if n > 1 and (topology == "full" or orc.is_global_step(k0 + j, H)):
            assert got[j] == 0.0
    if k0:
        assert np.isnan(trace.cpu().numpy()[:k0]).all()                # entries before k0 untouched
    sim.close()


@pytest.mark.parametrize("kind,n,d,M,B,topology,H,momentum,nesterov", [
    ("logreg", 20, 10, 100, 3, "ring", 1, 0.9, False), ("logreg", 20, 10, 100, 3, "ring", 0, 0.9, True),
    ("logreg", 20, 10, 100, 3, "expo1", 0, 0.0, False), ("logreg", 20, 10, 100, 3, "grid", 0, 0.9, False),
    ("logreg", 20, 10, 100, 3, "expo", 0, 0.9, True), ("logreg", 9, 17, 50, 2, "custom", 0, 0.5, False),
    ("lsq", 6, 40, 30, 0, "ring", 0, 0.9, False), ("lsq", 6, 40, 30, 7, "full", 0, 0.0, False)])
def test_one_iteration_from_a_random_state(hx, kind, n, d, M, B, topology, H, momentum, nesterov):
    seed = n + d + M
    sim, feat, tgt, grad, W = build(hx, kind, n, d, M, topology, H, momentum, nesterov, seed, small=True)
    X, Mb, _ = inputs.random_state(n, d, seed=seed, scale=0.3)
    for k in (0, 1, 2, 7):
        idx = inputs.batch_indices(1, n, B, M, seed=seed + k) if B else None
        sim.set_state(X=X, M=Mb, k=k)
        sim.run(1, sim.upload_batches(idx) if B else None)
        G = grad(feat, tgt, X, None if idx is None else idx[0])
        X_ref, M_ref = orc.gossip_pga_step(X, Mb if momentum else np.zeros_like(Mb), G.astype(np.float32), k,
                                           topology=topology, H=H, lr=float(np.float32(LR)), momentum=momentum,
                                           nesterov=nesterov, W=W)
        scale = max(np.abs(X_ref).max(), np.abs(X).max())
        assert np.abs(sim.X.cpu().numpy() - X_ref).max() <= TOL_STEP * scale, k
        if momentum:
            assert rel(sim.M.cpu().numpy(), M_ref) <= TOL_STEP, k
        assert rel(sim.G.cpu().numpy(), G) <= TOL_STEP, k
    sim.close()


def test_both_paths_of_gpga_run_agree_and_long_runs_are_chunked(hx):
    kind, n, d, M, B, T = "logreg", 20, 10, 500, 2, 700             # 700 iterations: three launches
    from paper_2105_09080_amd import binding as Bn
    idx = inputs.batch_indices(T, n, B, M, seed=9)
    out = []
    for small in (True, False):
        sim, feat, tgt, grad, _ = build(hx, kind, n, d, M, "ring", 16, 0.9, False, 9, small=small)
        Bn.gpga_lr_schedule_step(sim.ctx, LR, 250, 0.5)
        trace = sim.attach_trace(T)
        sim.run(T, sim.upload_batches(idx))
        out.append((sim.X.cpu().numpy(), sim.M.cpu().numpy(), trace.cpu().numpy(), sim.k, sim.lr))
        sim.close()
    (Xa, Ma, ta, ka, lra), (Xb, Mb, tb, kb, lrb) = out
    assert ka == kb == T and lra == lrb == pytest.approx(LR * 0.25)
    assert rel(Xa, Xb) <= TOL_FINAL and rel(Ma, Mb) <= TOL_FINAL
    assert np.abs(ta - tb).max() <= TOL_FINAL * np.linalg.norm(Xb)


def test_out_of_range_sample_index_poisons_only_its_node(hx):
    n, d, M, B = 6, 10, 20, 2
    sim, feat, tgt, grad, _ = build(hx, "logreg", n, d, M, "none", 0, 0.0, False, 5, small=True)
    idx = inputs.batch_indices(1, n, B, M, seed=5)
    idx[0, 3, 1] = M                                                   # one past the end
    X = inputs.random_state(n, d, seed=5, scale=0.3)[0]
    sim.set_state(X=X, k=0)
    sim.run(1, sim.upload_batches(idx))
    G, Xn = sim.G.cpu().numpy(), sim.X.cpu().numpy()
    assert np.isnan(G[3]).all() and np.isnan(Xn[3]).all()
    keep = [i for i in range(n) if i != 3]
    assert np.isfinite(G[keep]).all() and np.isfinite(Xn[keep]).all()
    sim.close()


def test_iteration_rate_on_the_simulation_shape(hx):
    # n = 100 nodes, d = 10, one sample per node and iteration (Sec. 5.1): both paths, for the record
    n, d, M, B, T = 100, 10, 2000, 1, 3000
    idx = inputs.batch_indices(T, n, B, M, seed=1)
    rates = {}
    for small in (True, False):
        sim, *_ = build(hx, "logreg", n, d, M, "ring", 16, 0.0, False, 1, small=small)
        idx_d = sim.upload_batches(idx)
        trace = sim.attach_trace(2 * T)
        sim.run(T, idx_d)
        torch.cuda.synchronize()
        sim.set_state(k=0)
        t0 = time.perf_counter()
        sim.run(T, idx_d)
        torch.cuda.synchronize()
        rates[small] = T / (time.perf_counter() - t0)
        assert (int(sim.query("step_path")) == 7) == small
        sim.close()
    # a figure for the record, not an assertion: wall-clock comparisons do not belong in a parity suite
    print(f"iterations/s: single-workgroup path {rates[True]:.0f}, kernel-per-stage path {rates[False]:.0f}")
