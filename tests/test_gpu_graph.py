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
    (64, 300_004, "expo1", {"blocks_per_cu": 2, "pace_gbs": 4000}),   # paced persistent launches inside the graph
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
    sim.close()
