"""GPU parity of the consensus trace (gpga_set_trace): the per-step consensus
distance recorded on the device, by the fused kernel where it stores whole
columns and by a reduction pass elsewhere, against the oracle's definition."""
import numpy as np
import pytest

from oracle import gpga_oracle as orc
from paper_2105_09080_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import harness
    return harness


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


# expect = (step_path, trace_fused) of the gossip steps as gpga_query reports them (None = any), None where the steps of a run
# differ among themselves (one-peer offsets) or the case is not about the path.  Paths: 1 stencil walk, 2 row-streaming
# one-peer kernel, 4 whole-tile sparse W, 5 sliding-window sparse W, 6 two passes.
CASES = [
    # n, d, topology, H, momentum, T, opts, expect
    (8, 600_000, "ring", 4, 0.9, 9, {}, (1, 1)),                      # one walker per column: sums ride along
    (64, 300_004, "ring", 6, 0.9, 8, {}, (1, 0)),                     # too few column tiles for one walker each: rows split
    (64, 300_004, "ring", 0, 0.0, 3, {"blocks_per_cu": 0}, (1, 0)),
    (64, 1_200_000, "ring", 3, 0.9, 4, {"blocks_per_cu": 4, "pace_gbs": 5000}, (1, 1)),   # persistent paced launch, fused sums
    (5, 1000, "ring", 3, 0.9, 7, {}, (1, 1)),                         # short cycle, one walker
    (5, 1000, "expo1", 3, 0.9, 7, {}, (1, 1)),                        # n odd: every one-peer offset is one cycle
    (64, 4100, "ring", 4, 0.9, 6, {}, (1, 0)),                        # rows split over wavefronts: reduction pass
    (64, 300_004, "expo1", 0, 0.9, 7, {}, None),                      # several cycles: reduction pass
    # paced one-peer steps on enough column tiles for one walker per cycle: a work item takes all cycles of its tile
    # (long cycles: the walk; cycles of 2 .. 16 rows: the row-streaming kernel), so its lanes store whole columns
    (64, 1_100_000, "expo1", 0, 0.9, 7, {"blocks_per_cu": 2, "pace_gbs": 4000}, (None, 1)),
    (64, 1_100_000, "expo1", 6, 0.9, 8, {"blocks_per_cu": 4, "pace_gbs": 9000, "unroll": 2}, (None, 1)),
    (24, 1_100_000, "expo1", 0, 0.9, 6, {"blocks_per_cu": 2, "pace_gbs": 4000, "pace_min_cycle": 2}, (None, 1)),   # n not a power of two: cycles of 3 rows
    (24, 1_100_000, "expo1", 0, 0.9, 5, {"blocks_per_cu": 2, "pace_gbs": 4000}, None),   # ... which are not paced by default: reduction pass at that offset
    (64, 600_000, "expo1", 0, 0.9, 7, {"blocks_per_cu": 2, "pace_gbs": 4000}, None),   # fewer tiles: cycles split over wavefronts at some offsets
    (16, 1003, "ring", 5, 0.9, 6, {}, (1, 0)),                        # ragged d: scalar tail -> reduction pass
    (20, 2000, "grid", 4, 0.9, 6, {}, (4, 1)),                        # sparse W, tile kernel: sums ride along
    (64, 300_004, "grid", 6, 0.9, 7, {}, (4, 1)),
    (64, 300_004, "expo", 0, 0.9, 4, {"blocks_per_cu": 2}, (4, 1)),   # workgroups striding over several tiles
    (64, 100_000, "grid", 0, 0.0, 3, {"mix_waves": 16}, (4, 1)),      # 16 wavefronts' sums fill the whole tile
    (32, 100_000, "expo", 0, 0.9, 3, {"mix_waves": 16}, (4, 0)),      # ... and do not fit here: reduction pass
    (12, 2000, "expo", 0, 0.9, 4, {}, (4, 0)),                        # tile smaller than the sums: reduction pass
    (64, 100_000, "grid", 0, 0.9, 3, {"mix_lane_bytes": 8}, (4, 0)),  # narrow lanes, more workgroups than partial slots: reduction pass
    (64, 100_000, "grid", 0, 0.9, 3, {"mix_lane_bytes": 8, "blocks_per_cu": 2}, (4, 1)),   # ... persistent: sums ride along
    (200, 60_000, "expo", 5, 0.9, 5, {"blocks_per_cu": 1}, (4, 1)),   # 4-byte lanes (tile of 200 rows), sums ride along
    (300, 2000, "grid", 5, 0.9, 6, {}, (4, 0)),                       # small problem, 4-byte lanes, one workgroup per tile
    (300, 2000, "grid", 5, 0.9, 6, {"mix_two_pass": 1}, (6, 0)),      # two-pass sparse W: reduction pass
    (128, 60_000, "grid", 4, 0.9, 6, {"mix_band": 1}, (5, 1)),        # sliding-window kernel, 16-byte lanes: sums ride along
    (128, 60_000, "grid", 0, 0.9, 4, {"mix_band": 1, "mix_lane_bytes": 8, "blocks_per_cu": 1}, (5, 1)),
    (128, 60_000, "grid", 0, 0.0, 4, {"mix_band": 1, "mix_lane_bytes": 4, "blocks_per_cu": 1}, (5, 1)),
    (128, 60_000, "grid", 0, 0.9, 3, {"mix_band": 1, "mix_lane_bytes": 4}, (5, 0)),   # more workgroups than slots: reduction pass
    (36, 30_000, "ring", 3, 0.9, 5, {"mix_band": 1}, None),           # (the ring stencil kernel; mix_band only matters for sparse W)
    (12, 500, "none", 3, 0.5, 5, {}, None),
]


@pytest.mark.parametrize("n,d,topology,H,momentum,T,opts,expect", CASES)
def test_trace_matches_the_oracles_consensus_distance(hx, n, d, topology, H, momentum, T, opts, expect):
    sim = hx.Simulation(n, d, topology=topology, H=H, lr=0.05, momentum=momentum)
    for name, v in opts.items():
        sim.set_option(name, v)
    sim.problem_synthetic(21, 1.0)
    trace = sim.attach_trace(T)
    want, norms = [], []
    for k in range(T):
        sim.local_grad()
        X_prev, M_prev, G_prev = host(sim.X), (host(sim.M) if momentum else None), host(sim.G)
        sim.step()
        if expect is not None and not orc.is_global_step(k, H):
            took = (int(sim.query("step_path")), int(sim.query("trace_fused")))
            assert all(e is None or e == t for e, t in zip(expect, took)), \
                f"step {k} ran as path {took[0]} with trace_fused {took[1]}, expected {expect}"
        X = host(sim.X)
        # the traced launches are also ordinary steps: one oracle step from the GPU's previous state
        X1, _ = orc.gossip_pga_step(X_prev, M_prev if momentum else np.zeros_like(X_prev), G_prev, k,
                                    topology=topology, H=H, lr=float(np.float32(0.05)), momentum=momentum)
        assert np.abs(X - X1).max() <= 1e-5 * np.abs(X1).max(), k
        want.append(orc.consensus_error(X))               # definition applied to the GPU's own iterate
        norms.append(np.linalg.norm(X))
        if orc.is_global_step(k, H):
            assert want[-1] == 0.0
    torch.cuda.synchronize()
    got = trace.cpu().numpy()
    for k in range(T):
        if orc.is_global_step(k, H):
            assert got[k] == 0.0, k
        else:
            assert abs(got[k] - want[k]) <= 1e-6 * want[k] + 1e-7 * norms[k], (k, got[k], want[k])
    # the synchronous entry point agrees with the last entry
    assert sim.consensus_error() == pytest.approx(got[T - 1], rel=1e-6, abs=1e-12)
    sim.close()


def test_trace_capacity_detach_and_free_running_oracle(hx):
    from paper_2105_09080_amd import binding as B
    n, d, T = 8, 600_000, 6
    sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.9)
    sim.problem_synthetic(3, 1e-3)
    trace = sim.attach_trace(4)                               # shorter than the run: later steps record nothing
    ref = orc.GossipPGA(n, 4096, topology="ring", H=0, lr=float(np.float32(0.1)), momentum=0.9, storage="f32")
    for k in range(T):
        sim.local_grad()
        sim.step()
    torch.cuda.synchronize()
    got = trace.cpu().numpy()
    assert np.isfinite(got).all() and (got > 0).all()
    # consensus distance grows with the random-walk of independent gradients: compare the
    # first steps with a free-running oracle on a column slab, scaled to the full width
    cols = np.arange(4096)
    for k in range(4):
        ref.step(orc.synthetic_grad(3, k, n, cols, 1e-3))
        assert got[k] == pytest.approx(orc.consensus_error(ref.X) * np.sqrt(d / 4096), rel=0.05)
    B.gpga_set_trace(sim.ctx, None, 0)
    before = trace.clone()
    sim.set_state(k=0)
    sim.local_grad()
    sim.step()
    torch.cuda.synchronize()
    assert torch.equal(before, trace)                         # detached: nothing is written
    with pytest.raises(B.GpgaError) as e:
        B.gpga_set_trace(sim.ctx, trace, 0)
    assert e.value.status == B.GPGA_EINVAL
    sim.close()
