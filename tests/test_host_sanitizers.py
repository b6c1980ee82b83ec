"""The library's host-only code (graph builders, validation of a caller's W, the beta estimate,
the schedule arithmetic of Algorithm 1, the controller of the pacing rate) built with AddressSanitizer + UndefinedBehaviorSanitizer
and run on the CPU: the sanitizers abort on any bad access or undefined operation, and the values
the program prints are compared with the oracle."""
import os
import subprocess

import numpy as np
import pytest

from oracle import gpga_oracle as orc

from paper_2105_09080_amd import build as gbuild


@pytest.fixture(scope="module")
def facts():
    exe = gbuild.build_host_check(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, f"host check failed (rc {res.returncode}):\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-4000:]
    return [line.split() for line in res.stdout.splitlines()]


def test_no_expectation_of_the_check_program_failed(facts):
    assert not [f for f in facts if f[0] == "FAIL"]
    assert ["failures", "0"] in facts
    rejected = [f for f in facts if f[0] == "rejected"]
    assert len(rejected) == 9 and all(f[2] != "ACCEPTED" for f in rejected)


def test_beta_of_the_named_graphs_matches_the_oracle(facts):
    checked = 0
    for f in facts:
        if f[0] != "beta":
            continue
        name, n, k, beta = f[1], int(f[2]), int(f[3]), float(f[4])
        if n > 200:
            continue                                   # dense eigenvalues in the oracle: keep it small
        ref = orc.beta_of(orc.mixing_matrix(name, n, k)) if n > 1 else 0.0
        assert beta == pytest.approx(ref, abs=2e-6), (name, n, k)
        checked += 1
    assert checked > 60
    # sizes the oracle's dense matrices cannot reach: the ring's closed form.  The estimate comes from a
    # Krylov space (it can only approach beta from below); at n = 1024 the space is large enough to resolve
    # the gap 1 - beta = 1.3e-5, at n = 2^20 (32 vectors, gap 1.2e-11) it is a lower bound and no more.
    ring = {int(f[2]): float(f[4]) for f in facts if f[0] == "beta" and f[1] == "ring"}
    closed = lambda n: (1 + 2 * np.cos(2 * np.pi / n)) / 3
    assert ring[1024] == pytest.approx(closed(1024), abs=1e-7)
    assert 0.999 < ring[1 << 20] <= closed(1 << 20) + 1e-9


def test_beta_of_random_doubly_stochastic_matrices_matches_the_oracle(facts):
    rows = [f for f in facts if f[0] == "random_w"]
    assert len(rows) == 8
    for f in rows:
        m = int(f[1])
        W = np.array([float(v) for v in f[2:2 + m * m]]).reshape(m, m)
        assert float(f[-1]) == pytest.approx(orc.beta_of(W), abs=5e-6)


def test_schedule_arithmetic_matches_the_oracle(facts):
    for f in facts:
        if f[0] == "tau":
            n, tau = int(f[1]), int(f[2])
            assert tau == orc.one_peer_tau(n)
            assert [int(v) for v in f[4:]] == [orc.one_peer_shift(n, k) for k in range(14)]
        if f[0] == "global_steps":
            H = int(f[1])
            assert [int(v) for v in f[2:]] == [k for k in range(100) if orc.is_global_step(k, H)]
    lr = {f[1]: [float(v) for v in f[2:]] for f in facts if f[0] == "lr"}
    f32 = lambda v: float(np.float32(v))
    assert lr["step"] == [pytest.approx(f32(orc.lr_step_decay(k, 0.2, 1000, 0.5)), rel=1e-7, abs=1e-30)
                          for k in (0, 999, 1000, 1999, 2000, 5000, 40000, 2000000)]
    assert lr["milestones"] == [pytest.approx(f32(orc.lr_warmup_milestones(k, 3.2, 500, 0.1, (3000, 6000, 9000), 0.1)), rel=1e-6)
                                for k in (0, 1, 250, 499, 500, 2999, 3000, 6000, 8999, 9000, 1000000)]
    assert lr["poly"] == [pytest.approx(f32(orc.lr_poly(k, 4e-3, 100, 1000, 0.5)), rel=1e-6, abs=1e-30)
                          for k in (0, 50, 100, 550, 999, 1000, 5000)]


def test_pacing_controller_finds_and_follows_the_edge_of_a_launch_model(facts):
    """The controller that sets the rate of paced launches, run on the CPU against a model of what a
    launch reports (keeps up below an edge rate with occasional late launches, falls behind above it):
    the check program asserts the settling time, the held rate and the reaction to a moved edge
    itself (FAIL lines); here the printed figures are looked at once more."""
    rows = [f for f in facts if f[0] == "pace_model"]
    assert len(rows) == 6
    for f in rows:
        v = dict(zip(f[2::2], f[3::2]))
        edge, mean = float(v["edge"]), float(v["mean_rate"])
        assert 0.985 * edge <= mean <= 1.012 * edge
        assert int(v["settle"]) <= 48 and int(v["drop_recover"]) <= 12
    assert [f for f in facts if f[0] == "pace_model_limit"]
