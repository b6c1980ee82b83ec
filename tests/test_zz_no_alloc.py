"""The entry point that allocates nothing (gpga_consensus_error_static) against
gpga_consensus_error, through the C ABI: two calls in a row, the second on a smaller
input, on aligned and unaligned rows; the size limit gives a clear error."""
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


def _state(n, d, seed):
    base = inputs.initial_point(d, seed=seed).astype(np.float64) * 10.0
    dev = inputs.random_state(n, d, seed=seed + 1, scale=1e-2)[0].astype(np.float64)
    return (base[None, :] + dev).astype(np.float32)


def test_static_scratch_consensus_error_matches_the_allocating_entry_point(hx):
    from oracle import gpga_oracle as orc
    out = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda")
    # first call: wide (thousands of partial sums); second: smaller input, fewer partials, so
    # stale partials of the first call sit behind the ones the second call writes
    shapes = [(64, 3_000_004, 0), (16, 70_001, 3), (5, 1000, 0), (1024, 20_000, 0)]
    for call, (n, d, pad) in enumerate(shapes):
        X = _state(n, d, seed=40 + call)
        sim = hx.Simulation(n, d, topology="ring", H=0, lr=0.1, momentum=0.0, ld=d + pad)
        sim.set_state(X=X)
        sim.consensus_error_static(out[call % 2:])
        ref = sim.consensus_error()                       # synchronises the stream
        got = float(out[call % 2].item())
        assert got == pytest.approx(ref, rel=1e-12), f"call {call}: static {got!r} vs allocating {ref!r}"
        assert abs(got - orc.consensus_error(X)) <= 1e-5 * orc.consensus_error(X)
        # and again on the same input: the array keeps the last call's contents
        sim.consensus_error_static(out[call % 2:])
        torch.cuda.synchronize()
        assert float(out[call % 2].item()) == got
        sim.close()


def test_static_scratch_after_steps_and_size_limit(hx):
    from paper_2105_09080_amd import binding as B
    n, d = 8, 4100
    sim = hx.Simulation(n, d, topology="ring", H=4, lr=0.1, momentum=0.9)
    sim.problem_synthetic(3, 1e-3)
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    for k in range(5):
        sim.local_grad()
        sim.step()
        sim.consensus_error_static(out)
        ref = sim.consensus_error()
        assert float(out.item()) == pytest.approx(ref, rel=1e-12, abs=0.0)
        if k == 3:
            assert float(out.item()) == 0.0               # right after a global average
    with pytest.raises(B.GpgaError):
        sim.consensus_error_static(None)
    sim.close()
    # beyond the static array: rejected before anything is launched (no buffers of that size are
    # needed: bind only records pointers, and the call fails on the size check)
    big_d = 140_000_000
    ctx = B.gpga_create(2, big_d, "ring", 0, 0.1, 0.0)
    t = torch.zeros(4, device="cuda")
    # fake but non-overlapping, aligned addresses: never dereferenced on this path
    base = 1 << 40
    span = 2 * big_d * 4
    B.gpga_bind(ctx, base, base + 2 * span, None, base + 4 * span, big_d)
    with pytest.raises(B.GpgaError) as e:
        B.gpga_consensus_error_static(ctx, out)
    assert e.value.status == B.GPGA_EINVAL and "static scratch" in str(e.value)
    B.gpga_destroy(ctx)
    del t
