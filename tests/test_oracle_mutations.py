"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy of
the oracle's source (a dropped term, a wrong sign or index, a transposed operand,
an off-by-one in a schedule) and runs the pin suites against the copy in a child
process: some pin must fail.  The mistakes are planted in the oracle only, on the
CPU; nothing here touches the HIP library.

Where the paper is silent the pins hold the stated reading in place (direction of
the one-peer edge, node-local momentum buffer, counter layout of the random
numbers): those cases are marked "reading".  One free choice is left out on
purpose: which counter word addresses the node shift of the virtual features.
"""
import os
import subprocess
import sys
import textwrap
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "gpga_oracle.py")
PIN_SUITES = ["tests/test_oracle_pins.py", "tests/test_oracle_optim_pins.py", "tests/test_oracle_topology_pins.py"]

# (name, text in the oracle, replacement)
MUTATIONS = [
    # schedule of Algorithm 1
    ("average when mod(k, H) = 0", "return H > 0 and (k + 1) % H == 0", "return H > 0 and k % H == 0"),
    ("tau = floor(log2 n)", "math.ceil(math.log2(n))", "math.floor(math.log2(n))"),
    ("one-peer offset k mod (tau+1)", "(1 << (k % one_peer_tau(n))) % n", "(1 << (k % (one_peer_tau(n) + 1))) % n"),
    # mixing matrices
    ("ring neighbours two apart", "for j in (i - 1, i, i + 1):", "for j in (i - 2, i, i + 2):"),
    ("ring without the self weight", "for j in (i - 1, i, i + 1):\n                W[i, j % n] += 1.0 / 3.0",
     "for j in (i - 1, i + 1):\n                W[i, j % n] += 1.0 / 2.0"),
    ("one-peer weights 1/3, 2/3", "W[i, i] += 0.5\n            W[i, (i + s) % n] += 0.5",
     "W[i, i] += 1.0 / 3.0\n            W[i, (i + s) % n] += 2.0 / 3.0"),
    ("grid diagonal neighbour", "(a, b - 1), (a, b + 1)):", "(a, b - 1), (a + 1, b + 1)):"),
    ("grid numbered a*r + b", "i = a * c + b\n", "i = a * r + b\n"),
    ("grid of the least square shape", "r = int(math.isqrt(n))\n    while n % r:\n        r -= 1",
     "r = 1"),
    ("static exponential offsets j+1", "W[i, (i + (1 << j)) % n]", "W[i, (i + j + 1) % n]"),
    ("static exponential weight 1/tau", "W[i, (i + (1 << j)) % n] += 1.0 / (tau + 1)",
     "W[i, (i + (1 << j)) % n] += 1.0 / tau"),
    ("W = I scaled", "W[np.arange(n), np.arange(n)] = 1.0", "W[np.arange(n), np.arange(n)] = 0.5"),
    ("beta without removing J", "np.linalg.norm(W - np.full((n, n), 1.0 / n), 2)", "np.linalg.norm(W, 2)"),
    ("beta as Frobenius norm", "np.linalg.norm(W - np.full((n, n), 1.0 / n), 2)",
     "np.linalg.norm(W - np.full((n, n), 1.0 / n), 'fro')"),
    # the iteration
    ("ascent instead of descent", "return X - lr * M_new, M_new", "return X + lr * M_new, M_new"),
    ("dampened momentum", "M_new = momentum * np.asarray(Mbuf, dtype=np.float64) + G",
     "M_new = momentum * np.asarray(Mbuf, dtype=np.float64) + (1.0 - momentum) * G"),
    ("momentum on the old buffer only", "return X - lr * M_new, M_new",
     "return X - lr * (momentum * np.asarray(Mbuf, dtype=np.float64) + 0.0 * G + (G if momentum == 0.0 else 0.0)), M_new"),
    ("Nesterov look-ahead with the old buffer", "return X - lr * (G + momentum * M_new), M_new",
     "return X - lr * (G + momentum * np.asarray(Mbuf, dtype=np.float64)), M_new"),
    ("Nesterov without the gradient term", "return X - lr * (G + momentum * M_new), M_new",
     "return X - lr * (momentum * M_new), M_new"),
    ("combine then adapt", "X_next = Wk @ Y\n    return X_next, M_new",
     "X_next = Wk @ np.asarray(X, dtype=np.float64) - (np.asarray(X, dtype=np.float64) - Y)\n    return X_next, M_new"),
    ("global mean of the old iterate", "xbar = Y.mean(axis=0)                       # (1/n)",
     "xbar = np.asarray(X, dtype=np.float64).mean(axis=0)  # (1/n)"),
    ("global step keeps the rows", "X_next = np.broadcast_to(xbar, Y.shape).copy()\n    else:",
     "X_next = 0.5 * (Y + xbar)\n    else:"),
    ("mix columns instead of rows", "X_next = Wk @ Y\n    return X_next, M_new",
     "X_next = (Y.T @ Wk[:Y.shape[1], :Y.shape[1]]).T if Y.shape[0] == Y.shape[1] else Wk @ Y[::-1]\n    return X_next, M_new"),
    ("transposed W", "X_next = Wk @ Y\n    return X_next, M_new", "X_next = Wk.T @ Y\n    return X_next, M_new"),
    ("reading: one-peer edge points the other way", "W[i, (i + s) % n] += 0.5", "W[i, (i - s) % n] += 0.5"),
    ("reading: static exponential edges point the other way", "W[i, (i + (1 << j)) % n]", "W[i, (i - (1 << j)) % n]"),
    ("reading: momentum buffer averaged with the iterate", "X_next = np.broadcast_to(xbar, Y.shape).copy()\n    else:",
     "X_next = np.broadcast_to(xbar, Y.shape).copy()\n        M_new = np.broadcast_to(M_new.mean(axis=0), Y.shape).copy()\n    else:"),
    ("reading: momentum buffer mixed with the iterate", "X_next = Wk @ Y\n    return X_next, M_new",
     "X_next = Wk @ Y\n    M_new = Wk @ M_new\n    return X_next, M_new"),
    ("mixing matrix of the next iteration", "mixing_matrix(topology, Y.shape[0], k)", "mixing_matrix(topology, Y.shape[0], k + 1)"),
    ("zero momentum keeps the old buffer", "M_new = G.copy()", "M_new = np.asarray(Mbuf, dtype=np.float64) + G"),
    ("grid with more rows than columns", "return r, n // r", "return n // r, r"),
    # the driver
    ("iteration counter stuck", "self.X, self.M = self._store(X_next), self._store(M_next)\n        self.k += 1",
     "self.X, self.M = self._store(X_next), self._store(M_next)\n        self.k += 0"),
    ("step size of the next iteration", "lr=self.lr_at(self.k)", "lr=self.lr_at(self.k + 1)"),
    ("only node 0 starts at x0", "self.X = np.tile(x0[None, :], (n, 1))",
     "self.X = np.tile(x0[None, :], (n, 1)) * (np.arange(n)[:, None] == 0)"),
    ("fp32 storage not rounding", "return _round_f32(a) if self.storage == \"f32\"",
     "return np.asarray(a, dtype=np.float64) if self.storage == \"f32\""),
    ("step size not stored as fp32", "return float(np.float32(lr)) if self.storage == \"f32\" else float(lr)", "return float(lr)"),
    # diagnostics
    ("consensus over the wrong axis", "D = X - X.mean(axis=0, keepdims=True)", "D = X - X.mean(axis=1, keepdims=True)"),
    ("consensus without the root", "return float(np.sqrt(np.sum(D * D)))", "return float(np.sum(D * D))"),
    ("consensus per node", "return float(np.sqrt(np.sum(D * D)))", "return float(np.sqrt(np.sum(D * D) / X.shape[0]))"),
    ("mean over columns", "return np.asarray(X, dtype=np.float64).mean(axis=0)",
     "return np.asarray(X, dtype=np.float64).mean(axis=1)"),
    # step-size schedules
    ("halving one iteration early", "return base * factor ** (k // period)", "return base * factor ** ((k + 1) // period)"),
    ("warm-up one iteration ahead", "(base - warmup_start) * (k / warmup_iters)", "(base - warmup_start) * ((k + 1) / warmup_iters)"),
    ("milestone one iteration late", "passed = sum(1 for m in milestones if k >= m)", "passed = sum(1 for m in milestones if k > m)"),
    ("polynomial decay from iteration 0", "(1.0 - (k - warmup_iters) / (total_iters - warmup_iters)) ** power",
     "(1.0 - k / total_iters) ** power"),
    ("polynomial power as a factor", "(total_iters - warmup_iters)) ** power", "(total_iters - warmup_iters)) * power"),
    # losses and gradients
    ("least squares without 1/|B|", "G[i] = Ai.T @ r / len(bi)", "G[i] = Ai.T @ r"),
    ("least squares residual sign", "r = Ai @ np.asarray(X[i], dtype=np.float64) - bi\n        G[i]",
     "r = bi - Ai @ np.asarray(X[i], dtype=np.float64)\n        G[i]"),
    ("least squares loss without the half", "out[i] = 0.5 * np.dot(r, r) / len(bi)", "out[i] = np.dot(r, r) / len(bi)"),
    ("logistic gradient sign", "coef = -yi * expit(-yi * z) / len(yi)", "coef = yi * expit(-yi * z) / len(yi)"),
    ("logistic sigma of the wrong sign", "coef = -yi * expit(-yi * z) / len(yi)", "coef = -yi * expit(yi * z) / len(yi)"),
    ("logistic gradient without the label", "coef = -yi * expit(-yi * z) / len(yi)", "coef = -expit(-yi * z) / len(yi)"),
    ("logistic loss sign", "np.mean(np.logaddexp(0.0, -yi * z))", "np.mean(np.logaddexp(0.0, yi * z))"),
    ("logistic loss summed", "np.mean(np.logaddexp(0.0, -yi * z))", "np.sum(np.logaddexp(0.0, -yi * z))"),
    ("virtual-feature gradient sign", "coef = -yi * expit(-yi * z) / len(m)", "coef = yi * expit(-yi * z) / len(m)"),
    ("virtual features without the node shift", "return mu + zeta", "return zeta"),
    ("virtual features kept in double", "Hc = virtual_features(seed, i, m, cols, mu_var).astype(np.float32).astype(np.float64)\n            z +=",
     "Hc = virtual_features(seed, i, m, cols, mu_var)\n            z +="),
    ("node shift drawn from the sample stream", "TAG_MU = 3", "TAG_MU = 2"),
    ("least squares loss over all rows", "out[i] = 0.5 * np.dot(r, r) / len(bi)", "out[i] = 0.5 * np.dot(r, r) / A.shape[1]"),
    ("least squares gradient over all rows", "G[i] = Ai.T @ r / len(bi)", "G[i] = Ai.T @ r / A.shape[1]"),
    ("logistic gradient over all rows", "coef = -yi * expit(-yi * z) / len(yi)", "coef = -yi * expit(-yi * z) / y.shape[1]"),
    # counter-based generator
    ("Philox multipliers swapped", "p0 = _PHILOX_M0 * c0\n        p1 = _PHILOX_M1 * c2", "p0 = _PHILOX_M1 * c0\n        p1 = _PHILOX_M0 * c2"),
    ("Philox seven rounds", "for _ in range(10):", "for _ in range(7):"),
    ("Philox key words swapped", "(hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0",
     "(hi1 ^ c1 ^ np.uint64(k1)), lo1, (hi0 ^ c3 ^ np.uint64(k0)), lo0"),
    ("Philox output words permuted", "(hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0",
     "lo1, (hi1 ^ c1 ^ np.uint64(k0)), lo0, (hi0 ^ c3 ^ np.uint64(k1))"),
    ("Philox Weyl constants swapped", "k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF\n        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF",
     "k0 = (k0 + _PHILOX_W1) & 0xFFFFFFFF\n        k1 = (k1 + _PHILOX_W0) & 0xFFFFFFFF"),
    ("Philox key not bumped", "k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF", "k0 = k0 & 0xFFFFFFFF"),
    ("uniform without the half offset", ".astype(np.float64) + 0.5) * (2.0 ** -23)", ".astype(np.float64)) * (2.0 ** -23)"),
    ("uniform from 24 bits", "(2.0 ** -23)", "(2.0 ** -24)"),
    ("Box-Muller radius without the 2", "ra = np.sqrt(-2.0 * np.log(u0))", "ra = np.sqrt(-1.0 * np.log(u0))"),
    ("Box-Muller half angle", "ta = 2.0 * np.pi * u1", "ta = np.pi * u1"),
    ("Box-Muller second pair reuses the first radius", "rb * np.cos(tb), rb * np.sin(tb)", "ra * np.cos(tb), ra * np.sin(tb)"),
    ("synthetic gradient scaled by the variance", "return math.sqrt(var) * z", "return var * z"),
    ("reading: counter words for column and node swapped", "philox4x32_10(c4, node, j, tag, k0, k1)",
     "philox4x32_10(node, c4, j, tag, k0, k1)"),
    ("seed halves swapped", "k0, k1 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF",
     "k1, k0 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF"),
    # Gossip-AGA
    ("AGA warm-up keeps only the last loss", "self.F_init = 0.5 * (self.F_init + F)", "self.F_init = F"),
    ("AGA period rounded down", "H_new = math.ceil(ratio * self.H_init)", "H_new = math.floor(ratio * self.H_init)"),
    ("AGA period from the current H", "H_new = math.ceil(ratio * self.H_init)", "H_new = math.ceil(ratio * self.H)"),
    ("AGA ratio inverted", "ratio = self.F_init / F if F > 0.0", "ratio = F / self.F_init if F > 0.0 and self.F_init > 0.0"),
    ("AGA warm-up one iteration longer", "if k < self.K_w:", "if k <= self.K_w:"),
    ("AGA counter not reset", "self.C = 0\n            xbar", "xbar"),
    ("AGA without the period cap", "self.H = int(min(max(H_new, 1), self.H_max))", "self.H = int(max(H_new, 1))"),
    ("AGA step size of the next iteration", "p.lr_at(k), p.momentum", "p.lr_at(k + 1), p.momentum"),
    ("AGA mixing matrix of the next iteration", "mixing_matrix(p.topology, p.n, k)", "mixing_matrix(p.topology, p.n, k + 1)"),
    ("AGA takes the largest loss instead of the node mean",
     "F = float(np.mean(np.asarray(p._store(losses), dtype=np.float64)))",
     "F = float(np.max(np.asarray(p._store(losses), dtype=np.float64)))"),
]

RUNNER = textwrap.dedent("""
    import importlib.util, sys
    sys.path.insert(0, {root!r})
    import oracle
    spec = importlib.util.spec_from_file_location("oracle.gpga_oracle", {path!r})
    mod = importlib.util.module_from_spec(spec)
    sys.modules["oracle.gpga_oracle"] = mod
    spec.loader.exec_module(mod)
    oracle.gpga_oracle = mod
    import pytest
    sys.exit(pytest.main({suites!r} + ["-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]))
""")


def run_pins_against(path):
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    code = RUNNER.format(root=ROOT, path=path, suites=PIN_SUITES)
    p = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return p.returncode, p.stdout[-2000:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    src = open(ORACLE).read()
    work = tmp_path_factory.mktemp("mutants")
    paths = {}
    for j, (name, old, new) in enumerate(MUTATIONS):
        assert src.count(old) >= 1, f"mutation {name!r}: its text is not in the oracle any more"
        p = work / f"mutant_{j}.py"
        p.write_text(src.replace(old, new, 1))
        paths[name] = str(p)
    clean = work / "clean.py"
    clean.write_text(src)
    paths["<unchanged>"] = str(clean)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = dict(zip(paths, pool.map(run_pins_against, paths.values())))
    return results


def test_unchanged_copy_passes_every_pin(outcomes):
    rc, out = outcomes["<unchanged>"]
    assert rc == 0, out


@pytest.mark.parametrize("name", [m[0] for m in MUTATIONS])
def test_planted_mistake_fails_a_pin(outcomes, name):
    rc, out = outcomes[name]
    assert rc == 1, f"no pin noticed: {name}\n{out}"      # 1 = tests failed (not a collection or usage error)
