"""HIP-graph capture of the library's launches: a captured trajectory replays to
exactly the eager result, several times, with eager work between the replays.
(The library enqueues kernels only: no memsets, no allocation once scratch has
been sized by a first eager iteration.)"""
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


@pytest.mark.parametrize("n,d,topology,opts", [
    (8, 1000, "ring", {}),
    (20, 515, "grid", {}),
    # paced persistent launches inside the graph (one walker per cycle and short cycles paced too, so that every gossip step is)
    (64, 300_004, "expo1", {"blocks_per_cu": 2, "pace_gbs": 4000, "row_split": 1, "pace_min_cycle": 2}),
])
def test_captured_trajectory_replays_to_the_eager_result(hx, n, d, topology, opts):
    M, Bsz, T, H = 30, 4, 12, 4                       # T even: x / x_new end in the roles they started in
    feat, y, _ = inputs.logreg_problem(n, d, M, seed=4)
    feat = (feat / np.sqrt(d)).astype(np.float32)
    idx = inputs.batch_indices(T, n, Bsz, M, seed=4)
    stream = torch.cuda.Stream()
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.1, momentum=0.9, stream=stream)
    for name, v in opts.items():
        sim.set_option(name, v)
    sim.problem_logreg(feat, y)
    idx_d = sim.upload_batches(idx)
    trace = sim.attach_trace(T)
    X0 = inputs.random_state(n, d, seed=4)[0]

    def restart():
        sim.set_state(X=X0, M=np.zeros((n, d), dtype=np.float32), k=0)

    with torch.cuda.stream(stream):
        restart()
        sim.run(T, idx_d)                             # eager; also sizes the library's scratch
        torch.cuda.synchronize()
        X_eager, M_eager, tr_eager = sim.X.clone(), sim.M.clone(), trace.clone()
        restart()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            sim.run(T, idx_d)
        torch.cuda.synchronize()
        for rep in range(3):
            restart()                                 # eager work (copies) between the replays
            trace.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            # after T (even) iterations the live X is the buffer it was at capture time
            assert torch.equal(sim._bufs[0][:, :d], X_eager), rep
            assert torch.equal(sim.M, M_eager), rep
            assert torch.equal(trace, tr_eager), rep
    if "pace_gbs" in opts:   # the eager run and the three replays: every gossip step was a paced launch each time
        kinds = ("peer_long", "peer_16", "peer_8", "peer_4", "cycles")
        paced = sum(sim.query(f"pace_launches:{k}{dr}") for k in kinds for dr in ("", "/1"))
        assert paced == 4 * sum(1 for k in range(T) if (k + 1) % H), paced
    sim.close()


def test_paced_launches_stay_paced_when_a_captured_graph_replays(hx):
    # The pacing state lives on the device and resets itself at the end of every launch, so a
    # replayed launch publishes a fresh start time like an eager one.  Evidence that does not
    # depend on timing: every replayed launch is counted by its controller, and the slowest
    # wavefront of the last one ended within a fraction of a millisecond of its last deadline
    # (against a stale start time it would be late by the whole time since capture).
    # The event times of replay and eager run are printed as well.
    c = inputs.CONFIGS["cfg3"]
    n, d, T = c["n"], c["d"], 20
    stream = torch.cuda.Stream()
    sim = hx.Simulation(n, d, topology="expo1", H=c["H"], lr=c["lr"], momentum=c["momentum"], stream=stream)
    sim.problem_synthetic(c["seed"], c["grad_var"])
    kinds = ("peer_long", "peer_16", "peer_8", "peer_4", "cycles")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    with torch.cuda.stream(stream):
        sim.tune(16)
        sim.set_state(k=0)
        sim.run(T)                                    # warm
        sim.set_state(k=0)
        ev[0].record()
        sim.run(T)
        ev[1].record()
        torch.cuda.synchronize()
        X_eager = sim.X.clone()                       # two eager runs: x / x_new are back in their roles
        eager_ms = ev[0].elapsed_time(ev[1])
        count = lambda k: sim.query(f"pace_launches:{k}") + sim.query(f"pace_launches:{k}/1")   # both directions
        before = {k: count(k) for k in kinds}
        sim.set_state(k=0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            sim.run(T)
        torch.cuda.synchronize()
        captured = {k: count(k) for k in kinds}
        assert captured == before                     # capture itself runs nothing
        graph.replay()                                # warm
        ev[2].record()
        graph.replay()
        ev[3].record()
        torch.cuda.synchronize()
        replay_ms = ev[2].elapsed_time(ev[3])
    after = {k: count(k) for k in kinds}
    per_kind = dict.fromkeys(kinds, 0)
    for k in range(T):                                # offsets 1, 2 | 4 | 8 | 16 | 32 on n = 64
        per_kind[("peer_long", "peer_long", "peer_16", "peer_8", "peer_4", "cycles")[k % 6]] += 1
    for kind in kinds:
        assert after[kind] - captured[kind] == 2 * per_kind[kind], (kind, captured, after)
        for d in ("", "/1"):
            late, plan = sim.query(f"pace_last_late_us:{kind}{d}"), sim.query(f"pace_last_plan_us:{kind}{d}")
            assert plan > 1000.0 and late < 0.1 * plan, f"{kind}{d}: ended {late:.0f} us after its last deadline (plan {plan:.0f} us)"
    # reported, not asserted (a wall-clock comparison): unpaced launches would take about 1.19 x as long
    print(f"cfg3-shaped {T}-step trajectory: eager {eager_ms:.2f} ms, graph replay {replay_ms:.2f} ms")
    sim.close()
