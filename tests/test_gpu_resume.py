"""Checkpoint / resume and run-to-run reproducibility through the C ABI: the state
of a run is (X, M, k) plus the seeds, gradients and minibatches are addressed by
the iteration counter, so a run resumed at step k continues bit for bit."""
import numpy as np
import pytest

from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import harness
    return harness


def _run(hx, n, d, topology, H, T, start=None, nesterov=False, trace_len=0):
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.05, momentum=0.9)
    if nesterov:
        sim.set_nesterov(True)
    from paper_2105_09080_amd import binding as B
    B.gpga_lr_schedule_step(sim.ctx, float(np.float32(0.05)), 5, 0.5)
    sim.problem_synthetic(17, 1e-2)
    k0 = 0
    if start is not None:
        X, M, k0 = start
        sim.set_state(X=X, M=M, k=k0)
    trace = sim.attach_trace(trace_len) if trace_len else None
    for _ in range(k0, T):
        sim.local_grad()
        sim.step()
    torch.cuda.synchronize()
    out = (sim.X.cpu().numpy().copy(), sim.M.cpu().numpy().copy(), sim.k,
           None if trace is None else trace.cpu().numpy().copy())
    sim.close()
    return out


@pytest.mark.parametrize("n,d,topology,nesterov", [(64, 300_004, "ring", False), (64, 300_004, "expo1", True),
                                                   (20, 1003, "grid", False), (1024, 2052, "expo", False),
                                                   (16, 4100, "ring", True)])
def test_resumed_run_continues_bit_for_bit(hx, n, d, topology, nesterov):
    H, T, T1 = 6, 14, 8
    Xa, Ma, ka, tra = _run(hx, n, d, topology, H, T, nesterov=nesterov, trace_len=T)
    X1, M1, k1, _ = _run(hx, n, d, topology, H, T1, nesterov=nesterov)
    assert k1 == T1
    Xb, Mb, kb, trb = _run(hx, n, d, topology, H, T, start=(X1, M1, T1), nesterov=nesterov, trace_len=T)
    assert ka == kb == T
    assert np.array_equal(Xa, Xb) and np.array_equal(Ma, Mb)
    assert np.array_equal(tra[T1:], trb[T1:])                 # trace entries of the resumed steps too
    assert np.isnan(trb[:T1]).all()                           # earlier entries are not touched
    # and a second uninterrupted run reproduces the first exactly
    Xc, Mc, _, trc = _run(hx, n, d, topology, H, T, nesterov=nesterov, trace_len=T)
    assert np.array_equal(Xa, Xc) and np.array_equal(Ma, Mc) and np.array_equal(tra, trc)


@pytest.mark.parametrize("problem", ["lsq", "logreg", "synthetic"])
def test_run_equals_stepping_one_iteration_at_a_time(hx, problem):
    from paper_2105_09080_amd import binding as B
    n, d, M, Bsz, T, H = 8, 1003, 40, 6, 23, 4
    sims = []
    for _ in range(2):
        sim = hx.Simulation(n, d, topology="expo1", H=H, lr=0.02, momentum=0.9)
        idx_d = None
        if problem == "lsq":
            A, b, _ = inputs.lsq_problem(n, d, M, seed=2)
            sim.problem_lsq(A, b)
        elif problem == "logreg":
            feat, y, _ = inputs.logreg_problem(n, d, M, seed=2)
            sim.problem_logreg((feat / np.sqrt(d)).astype(np.float32), y)
            idx_d = sim.upload_batches(inputs.batch_indices(T, n, Bsz, M, seed=2))
        else:
            sim.problem_synthetic(5, 1e-2)
        sims.append((sim, idx_d))
    (a, idx_a), (b_, idx_b) = sims
    for k in range(T):
        a.local_grad(None if idx_a is None else idx_a[k])
        a.step()
    b_.run(10, idx_b)                                    # two calls: the table advances with the caller's slice
    b_.run(T - 10, None if idx_b is None else idx_b[10:])
    torch.cuda.synchronize()
    assert a.k == b_.k == T
    assert torch.equal(a.X, b_.X) and torch.equal(a.M, b_.M)
    b_.run(0, idx_b)                                     # zero iterations: nothing happens
    assert b_.k == T
    with pytest.raises(B.GpgaError) as e:
        B.gpga_run(b_.ctx, -1, None, 0)
    assert e.value.status == B.GPGA_EINVAL
    a.close(), b_.close()


def test_run_with_adaptive_averaging_equals_explicit_aga_steps(hx):
    n, d, M, Bsz, T = 16, 512, 64, 8, 60
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=21)
    feat = (feat / np.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, Bsz, M, seed=21)
    sims = []
    for _ in range(2):
        sim = hx.Simulation(n, d, topology="expo1", H=0, lr=0.5, momentum=0.9)
        sim.problem_logreg(feat, y)
        sim.aga_enable(2, 8, 12)
        sims.append((sim, sim.upload_batches(idx)))
    (a, idx_a), (b_, idx_b) = sims
    periods = []
    for k in range(T):
        loss = a.local_loss(idx_a[k])
        a.local_grad(idx_a[k])
        a.aga_step(loss)
        periods.append(a.period)
    b_.run(25, idx_b)
    b_.run(T - 25, idx_b[25:])
    torch.cuda.synchronize()
    assert b_.k == T and b_.period == periods[-1]
    assert len(set(periods)) >= 2                      # the period did adapt along the way
    assert torch.equal(a.X, b_.X) and torch.equal(a.M, b_.M)
    a.close(), b_.close()


def test_virtual_feature_gradient_is_reproducible_bit_for_bit(hx):
    # margins are combined from per-chunk partials in a fixed order (no floating-point atomics)
    n, d, M, Bsz = 8, 200_000, 50, 16
    y = inputs.virtual_labels(n, M, seed=3)
    idx = inputs.batch_indices(1, n, Bsz, M, seed=3)
    X = inputs.random_state(n, d, seed=3)[0]
    outs = []
    for _ in range(3):
        sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0)
        sim.problem_logreg_virtual(3, y, 0.5)
        idx_d = sim.upload_batches(idx)
        sim.set_state(X=X)
        sim.local_grad(idx_d[0])
        loss = sim.local_loss(idx_d[0])
        torch.cuda.synchronize()
        outs.append((sim.G.clone(), loss.clone()))
        sim.close()
    for G, loss in outs[1:]:
        assert torch.equal(G, outs[0][0]) and torch.equal(loss, outs[0][1])
