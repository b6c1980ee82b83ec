"""Seeded random sweeps against the CPU oracle, through the C ABI.

Steps: valid step configurations (shape, padding, topology, momentum,
averaging period, iteration counter, launch options, consensus trace) against the CPU
oracle, through the C ABI.  Every case checks two consecutive steps: iterates, momentum,
what happens to g, untouched padding columns, consensus distance (call and trace), node
mean, and identical rows after a global average.

Gradients: the four problems (least squares, logistic, logistic with regenerated
features, counter-addressed synthetic) over random n, d, M, minibatch sizes (0 = full
batch), padding and iteration counters: gradient, minibatch loss, untouched x and padding.

Runs: T iterations of the whole loop on synthetic gradients (a linear map of the draws, so
free-running trajectories stay comparable) over random topologies, periods, momentum forms,
step-size schedules and starting counters, driven by one gpga_run, two, or explicit
gradient + step calls: final iterate, momentum, iteration counter and the per-step
consensus trace."""
import math
import json

import numpy as np
import pytest

from oracle import gpga_oracle as orc
from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
SENTINEL = 12345.0
LR = float(np.float32(0.3))

N_CHOICES = [1, 2, 3, 4, 5, 7, 8, 12, 16, 20, 31, 32, 33, 48, 63, 64, 65, 100, 128, 129, 200, 256, 257, 300, 1024]
D_CHOICES = [1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 1000, 1023, 1024, 1025, 4096, 4100, 10_000, 65_536, 65_540,
             100_001, 300_004, 1_000_000]
OPTION_CHOICES = (("unroll", [1, 2, 4, 8]), ("waves", [1, 2, 4, 8]), ("row_split", [1, 2, 4, 8]), ("row_lanes", [1, 2, 4]),
                  ("xcd_swizzle", [0, 1]), ("blocks_per_cu", [0, 1, 2, 4, 8]), ("pace_gbs", [0, 2000, 6000, 16000]),
                  ("cycle_kernel", [0, 1]), ("pace_min_cycle", [2, 4, 8, 64]), ("mix_two_pass", [0, 1]), ("mix_band", [-1, 0, 1]), ("mix_tile_kb", [0, 64, 160]), ("mix_spmm_lanes", [0, 64, 128, 256]),
                  ("mix_waves", [2, 4, 8, 16]), ("mix_lane_bytes", [4, 8, 16]), ("mix_csr_lds", [0, 1]))


@pytest.fixture(scope="module")
def hx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import harness
    return harness


def draw_case(rng):
    def pick(xs):
        return xs[int(rng.integers(len(xs)))]
    n = int(pick(N_CHOICES))
    d = max(1, min(int(pick(D_CHOICES)), 3_000_000 // n))          # keeps the dense oracle quick
    mu = float(pick([0.0, 0.5, 0.9]))
    case = dict(n=n, d=d, pad=int(pick([0, 0, 0, 1, 2, 3, 4, 8, 13])),
                topology=pick(["ring", "expo1", "none", "full", "grid", "expo", "custom"]), momentum=mu,
                nesterov=bool(mu > 0 and rng.random() < 0.3), H=int(pick([0, 0, 1, 2, 3, 5])),
                k=int(pick([0, 1, 2, 3, 4, 5, 6, 7, 11, 12345])), options={}, trace=bool(rng.random() < 0.5),
                terms=int(pick([1, 3, 6])))
    if rng.random() < 0.7:
        for name, values in OPTION_CHOICES:
            if rng.random() < 0.35:
                case["options"][name] = int(pick(values))
    return case


def random_doubly_stochastic(n, terms, rng):
    w = rng.random(terms + 1)
    w /= w.sum()
    W = w[0] * np.eye(n)
    for t in range(terms):
        W += w[t + 1] * np.eye(n)[rng.permutation(n)]
    return W.astype(np.float32).astype(np.float64)


def check_case(hx, case, seed, rng):
    from paper_2105_09080_amd import binding as B
    n, d, topology, mu, H, k = case["n"], case["d"], case["topology"], case["momentum"], case["H"], case["k"]
    nesterov = case["nesterov"]
    X, Mb, G = inputs.random_state(n, d, seed=seed)
    W = random_doubly_stochastic(n, case["terms"], rng) if topology == "custom" else None
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.3, momentum=mu, ld=d + case["pad"])
    buffers = sim._bufs + [sim.g] + ([sim.m] if sim.m is not None else [])
    for t in buffers:
        t.fill_(SENTINEL)
    torch.cuda.synchronize()
    if W is not None:
        sim.set_mixing(W)
    if nesterov:
        sim.set_nesterov(True)
    applied = {}
    for name, v in case["options"].items():
        try:
            sim.set_option(name, v)
            applied[name] = v
        except B.GpgaError:                       # a combination the library refuses (row_split > waves)
            pass
    trace = sim.attach_trace(k + 4) if case["trace"] else None
    sim.set_state(X=X, M=Mb, G=G, k=k)
    X_ref = X.astype(np.float64)
    M_ref = (Mb if mu else np.zeros_like(Mb)).astype(np.float64)
    G_now = G.astype(np.float64)
    problems = []
    for j in range(2):
        is_global = orc.is_global_step(k + j, H)
        sparse = topology in ("grid", "expo", "custom") and n > 1 and not is_global
        sim.step()
        Y_ref, _ = orc.local_update(X_ref, M_ref, G_now, LR, mu, nesterov)
        X_next, M_next = orc.gossip_pga_step(X_ref, M_ref, G_now, k + j, topology=topology, H=H, lr=LR, momentum=mu,
                                             nesterov=nesterov, W=W)
        X_ref = X_next.astype(np.float32).astype(np.float64)
        M_ref = M_next.astype(np.float32).astype(np.float64)
        # a few ulp of the step's input scale (a global average at d = 1 can cancel to nearly 0)
        scale = max(np.abs(X_ref).max(), np.abs(Y_ref).max(), 1e-30)
        X_gpu = sim.X.cpu().numpy().astype(np.float64)
        err = {"X": np.abs(X_gpu - X_ref).max() / scale}
        if mu:
            err["M"] = np.abs(sim.M.cpu().numpy() - M_ref).max() / max(np.abs(M_ref).max(), 1e-30)
        G_gpu = sim.G.cpu().numpy().astype(np.float64)
        if not np.array_equal(G_gpu, G_now):       # on every path the gradients are only read
            problems.append(f"step {j}: g was modified")
        if not all(bool((t[:, d:] == SENTINEL).all().item()) for t in buffers):
            problems.append(f"step {j}: padding columns were written")
        norm = np.linalg.norm(X_ref) + 1e-30
        ce_ref = orc.consensus_error(X_ref)
        err["consensus"] = abs(sim.consensus_error() - ce_ref) / norm
        if trace is not None:
            err["trace"] = abs(float(trace[k + j].item()) - ce_ref) / norm
        err["mean"] = np.abs(sim.mean().cpu().numpy() - orc.node_mean(X_ref)).max() / scale
        if is_global or topology == "full":
            rows = sim.X.cpu().numpy()
            if not all(np.array_equal(rows[0], rows[i]) for i in range(n)):
                problems.append(f"step {j}: rows differ after a global average")
        problems += [f"step {j}: {what} off by {e:.3e}" for what, e in err.items() if not e <= TOL]
    sim.close()
    return problems


@pytest.mark.parametrize("seed", [101, 202, 303, 404])
def test_random_valid_configurations_match_the_oracle(hx, seed):
    rng = np.random.default_rng(seed)
    failures = []
    for j in range(150):
        case = draw_case(rng)
        print("case", seed, j, json.dumps(case), flush=True)       # names the case should a launch go wrong
        problems = check_case(hx, case, seed * 1000 + j, rng)
        if problems:
            failures.append((j, case, problems))
    assert not failures, failures[:5]


def check_gradient_case(hx, case, seed):
    prob, n, d, M, Bsz, k = case["problem"], case["n"], case["d"], case["M"], case["B"], case["k"]
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0, ld=d + case["pad"])
    buffers = sim._bufs + [sim.g]
    for t in buffers:
        t.fill_(SENTINEL)
    torch.cuda.synchronize()
    X = inputs.random_state(n, d, seed=seed, scale=case["x_scale"])[0]
    sim.set_state(X=X, k=k)
    idx = inputs.batch_indices(1, n, Bsz, M, seed=seed + 1)[0] if Bsz else None
    loss = loss_ref = None
    if prob == "synthetic":
        sim.problem_synthetic(seed, 1e-3)
        sim.local_grad()
        G_ref = orc.synthetic_grad(seed, k, n, np.arange(d), 1e-3)
    elif prob == "virtual":
        y = inputs.virtual_labels(n, M, seed)
        sim.problem_logreg_virtual(seed, y, 0.5)
        sim.local_grad(sim.upload_batches(idx))
        G_ref = orc.logreg_virtual_grad(seed, y, X, idx, 0.5)
    else:
        make, attach, grad, loss_of = {
            "lsq": (inputs.lsq_problem, sim.problem_lsq, orc.lsq_grad, orc.lsq_loss),
            "logreg": (inputs.logreg_problem, sim.problem_logreg, orc.logreg_grad, orc.logreg_loss)}[prob]
        data, target, _ = make(n, d, M, seed=seed)
        attach(data, target)
        idx_d = sim.upload_batches(idx) if Bsz else None
        sim.local_grad(idx_d)
        loss = sim.local_loss(idx_d).cpu().numpy().astype(np.float64)
        G_ref, loss_ref = grad(data, target, X, idx), loss_of(data, target, X, idx)
    problems = []
    e = np.abs(sim.G.cpu().numpy() - G_ref).max() / max(np.abs(G_ref).max(), 1e-30)
    if not e <= TOL:
        problems.append(f"gradient off by {e:.3e}")
    if loss_ref is not None:
        e = np.abs(loss - loss_ref).max() / max(np.abs(loss_ref).max(), 1e-30)
        if not e <= TOL:
            problems.append(f"loss off by {e:.3e}")
    if not all(bool((t[:, d:] == SENTINEL).all().item()) for t in buffers):
        problems.append("padding columns were written")
    if not np.array_equal(sim.X.cpu().numpy(), X):
        problems.append("x was modified")
    sim.close()
    return problems


def draw_gradient_case(rng):
    def pick(xs):
        return xs[int(rng.integers(len(xs)))]
    prob = pick(["lsq", "logreg", "virtual", "synthetic"])
    n = int(pick([1, 2, 3, 5, 8, 17, 32, 64]))
    d = int(pick([1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 1000, 1023, 1025, 4096, 4099, 10_000, 20_000, 65_540]))
    M = int(pick([1, 2, 7, 20, 33, 64, 100]))
    Bsz = int(pick([0, 1, 2, 6, 16, 32, 33, 50]))
    x_scale = 1.0
    if prob == "virtual":                          # needs an explicit minibatch of at most 32 samples
        Bsz, d = min(max(Bsz, 1), 32), min(d, 20_000)
        x_scale = 1.0 / math.sqrt(d)
    elif prob == "logreg":
        x_scale = float(pick([1.0, 0.3, 0.01, 30.0]))
    if prob in ("lsq", "logreg"):
        while n * M * d > 4_000_000:               # keeps the feature array small
            if M > 7:
                M = max(1, M // 2)
            else:
                d = max(1, d // 2)
    return dict(problem=prob, n=n, d=d, M=M, B=Bsz, pad=int(pick([0, 0, 1, 3, 4])), k=int(pick([0, 1, 7, 123456])),
                x_scale=x_scale)


@pytest.mark.parametrize("seed", [11, 22])
def test_random_gradient_configurations_match_the_oracle(hx, seed):
    rng = np.random.default_rng(seed)
    failures = []
    for j in range(250):
        case = draw_gradient_case(rng)
        print("gradient case", seed, j, json.dumps(case), flush=True)
        problems = check_gradient_case(hx, case, seed * 1000 + j)
        if problems:
            failures.append((j, case, problems))
    assert not failures, failures[:5]


def check_run_case(hx, case, seed):
    from paper_2105_09080_amd import binding as B
    n, d, T, k0, mu = case["n"], case["d"], case["T"], case["k0"], case["momentum"]
    base, var = 0.2, 1e-1
    f32 = lambda v: float(np.float32(v))
    x0 = inputs.initial_point(d, seed=seed)
    sim = hx.Simulation(n, d, topology=case["topology"], H=case["H"], lr=base, momentum=mu, x0=x0)
    if case["nesterov"]:
        sim.set_nesterov(True)
    if case["schedule"] == "step":
        B.gpga_lr_schedule_step(sim.ctx, base, 4, 0.5)
        lr = lambda k: orc.lr_step_decay(k, f32(base), 4, 0.5)
    elif case["schedule"] == "milestones":
        B.gpga_lr_schedule_milestones(sim.ctx, base, 3, 0.05, [6, 11], 0.1)
        lr = lambda k: orc.lr_warmup_milestones(k, f32(base), 3, f32(0.05), [6, 11], f32(0.1))
    elif case["schedule"] == "poly":
        B.gpga_lr_schedule_poly(sim.ctx, base, 2, 30, 2.0)
        lr = lambda k: orc.lr_poly(k, f32(base), 2, 30, 2.0)
    else:
        lr = base
    sim.problem_synthetic(seed, var)
    ref = orc.GossipPGA(n, d, topology=case["topology"], H=case["H"], lr=lr, momentum=mu, nesterov=case["nesterov"],
                        x0=x0.astype(np.float32), storage="f32")
    ref.k = k0
    B.gpga_set_iter(sim.ctx, k0)
    trace = sim.attach_trace(k0 + T)
    if case["driver"] == "run":
        sim.run(T)
    elif case["driver"] == "two runs":
        sim.run(T // 2)
        sim.run(T - T // 2)
    else:
        for _ in range(T):
            sim.local_grad()
            sim.step()
    consensus = []
    for j in range(T):
        ref.step(orc.synthetic_grad(seed, k0 + j, n, np.arange(d), var))
        consensus.append(orc.consensus_error(ref.X))
    err = {"X": np.abs(sim.X.cpu().numpy() - ref.X).max() / max(np.abs(ref.X).max(), 1e-30)}
    if mu:
        err["M"] = np.abs(sim.M.cpu().numpy() - ref.M).max() / max(np.abs(ref.M).max(), 1e-30)
    err["trace"] = np.abs(trace.cpu().numpy()[k0:k0 + T] - np.array(consensus)).max() / (np.linalg.norm(ref.X) + 1e-30)
    problems = [f"{what} off by {e:.3e}" for what, e in err.items() if not e <= 1e-4]
    if sim.k != k0 + T:
        problems.append(f"iteration counter {sim.k}, expected {k0 + T}")
    sim.close()
    return problems


@pytest.mark.parametrize("seed", [7, 8])
def test_random_runs_match_the_oracle_driver(hx, seed):
    rng = np.random.default_rng(seed)

    def pick(xs):
        return xs[int(rng.integers(len(xs)))]
    failures = []
    for j in range(200):
        n = int(pick([1, 2, 3, 5, 8, 12, 16, 20, 33, 64, 100, 257]))
        mu = float(pick([0.0, 0.5, 0.9]))
        case = dict(n=n, d=max(1, min(int(pick([1, 3, 4, 64, 257, 1000, 1024, 4100, 20_000])), 400_000 // n)),
                    topology=pick(["ring", "expo1", "none", "full", "grid", "expo"]), momentum=mu,
                    nesterov=bool(mu > 0 and rng.random() < 0.4), H=int(pick([0, 1, 2, 3, 4, 7])),
                    T=int(pick([1, 2, 5, 9, 16, 25])), k0=int(pick([0, 0, 3, 10])),
                    schedule=pick(["constant", "step", "milestones", "poly"]), driver=pick(["run", "two runs", "calls"]))
        print("run case", seed, j, json.dumps(case), flush=True)
        problems = check_run_case(hx, case, seed * 1000 + j)
        if problems:
            failures.append((j, case, problems))
    assert not failures, failures[:5]
