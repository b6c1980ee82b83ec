"""CPU-side checks of the C ABI: the built library loads, exports every symbol
that include/gpga.h declares, the Python binding covers the same set, and
argument validation that happens before any device call behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gpga.h")
LIB = os.path.join(ROOT, "paper_2105_09080_amd", "libgpga.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gpga_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} has not been built (run __graft_entry__.build())")
    return ctypes.CDLL(LIB)


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("gpga_create", "gpga_destroy", "gpga_bind", "gpga_local_grad", "gpga_step",
                 "gpga_consensus_error", "gpga_mean"):
        assert must in names
    assert len(names) >= 20


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"libgpga.so does not export {name}"


def test_binding_covers_exactly_the_declared_symbols():
    from paper_2105_09080_amd import binding
    bound = sorted(name for name, _, _ in binding.SIGNATURES)
    assert bound == declared_functions()
    for name in bound:                      # one Python function per entry point, same name
        assert callable(getattr(binding, name))
    assert binding.gpga_version().startswith("libgpga")


def test_create_rejects_bad_arguments_before_touching_the_device(lib):
    from paper_2105_09080_amd import binding as B
    out = ctypes.c_void_p()
    create = lambda *a: B.raw_status("gpga_create", ctypes.byref(out), *a)
    ok_args = dict(n=4, d=16, topo=0, H=2, lr=0.1, mu=0.9)

    def call(**kw):
        a = dict(ok_args)
        a.update(kw)
        return create(a["n"], a["d"], a["topo"], a["H"], a["lr"], a["mu"])

    assert call(n=0) == B.GPGA_EINVAL
    assert call(n=-3) == B.GPGA_EINVAL
    assert call(d=0) == B.GPGA_EINVAL
    assert call(topo=7) == B.GPGA_EINVAL
    assert call(topo=-1) == B.GPGA_EINVAL
    assert call(H=-1) == B.GPGA_EINVAL
    assert call(lr=float("inf")) == B.GPGA_EINVAL
    assert call(lr=float("nan")) == B.GPGA_EINVAL
    assert call(lr=-0.1) == B.GPGA_EINVAL
    assert call(mu=1.0) == B.GPGA_EINVAL
    assert call(mu=-0.1) == B.GPGA_EINVAL
    assert out.value is None
    assert B.raw_status("gpga_create", None, 4, 16, 0, 2, 0.1, 0.9) == B.GPGA_EINVAL


def test_null_context_is_rejected_everywhere(lib):
    from paper_2105_09080_amd import binding as B
    assert B.raw_status("gpga_step", None) == B.GPGA_EINVAL
    assert B.raw_status("gpga_destroy", None) == B.GPGA_EINVAL
    assert B.raw_status("gpga_set_lr", None, 0.1) == B.GPGA_EINVAL
    assert B.raw_status("gpga_local_grad", None, None, 0) == B.GPGA_EINVAL
    assert B.raw_status("gpga_iter", None) == -1
    assert B.gpga_last_error(None) == "null context"


def test_workload_table_matches_the_stated_configurations():
    from paper_2105_09080_amd import inputs
    c = inputs.CONFIGS
    assert (c["cfg1"]["n"], c["cfg1"]["d"], c["cfg1"]["H"], c["cfg1"]["T"]) == (8, 1000, 4, 200)
    assert (c["cfg2"]["n"], c["cfg2"]["d"], c["cfg2"]["B"], c["cfg2"]["H"], c["cfg2"]["T"]) == (32, 10_000, 32, 16, 500)
    assert (c["cfg3"]["n"], c["cfg3"]["d"], c["cfg3"]["H"]) == (64, 25_600_000, 48)
    assert (c["cfg4"]["n"], c["cfg4"]["d"], c["cfg4"]["H"]) == (64, 110_000_000, 6)
    assert (c["cfg5"]["n"], c["cfg5"]["d"], c["cfg5"]["M"], c["cfg5"]["B"]) == (1024, 1_000_000, 500, 16)
    assert set(c["cfg5"]["H_sweep"]) == {1, 8, 64, 0}


def test_input_generators_are_seeded_and_shaped():
    import numpy as np
    from paper_2105_09080_amd import inputs
    A, b, xs = inputs.lsq_problem(3, 20, 5, seed=4)
    A2, b2, _ = inputs.lsq_problem(3, 20, 5, seed=4)
    assert A.shape == (3, 5, 20) and b.shape == (3, 5) and A.dtype == np.float32
    assert np.array_equal(A, A2) and np.array_equal(b, b2)
    assert not np.array_equal(A, inputs.lsq_problem(3, 20, 5, seed=5)[0])
    feat, y, _ = inputs.logreg_problem(2, 30, 7, seed=1)
    assert feat.shape == (2, 7, 30) and set(np.unique(y)) <= {-1.0, 1.0}
    idx = inputs.batch_indices(4, 3, 6, 9, seed=2)
    assert idx.shape == (4, 3, 6) and idx.dtype == np.int32 and idx.min() >= 0 and idx.max() < 9
    yv = inputs.virtual_labels(5, 11, seed=0)
    assert yv.shape == (5, 11) and set(np.unique(yv)) <= {-1.0, 1.0}
    cols = inputs.slab_columns(1000, 4, 16)
    assert cols[0] == 0 and cols[-1] == 999 and len(cols) == 64 and (np.diff(cols) > 0).all()


# ---- host-side graph logic (no device involved) ---------------------------------------------

def _dense_to_csr(W):
    import numpy as np
    rows, cols = np.nonzero(W)
    ptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=W.shape[0]))])
    return ptr, cols, W[rows, cols].astype(np.float32)


def test_topology_beta_reproduces_the_values_printed_in_the_paper(lib):
    from conftest import read_golden
    from paper_2105_09080_amd import binding as B
    for n_s, beta_s in read_golden("ring_beta.txt"):          # Sec. 5.1: ring, n = 20, 50, 100
        assert abs(B.gpga_topology_beta("ring", int(n_s)) - float(beta_s)) < 1e-3


@pytest.mark.parametrize("topology", ["ring", "grid", "expo", "expo1", "none", "full"])
@pytest.mark.parametrize("n", [1, 2, 3, 7, 20, 50, 64, 100, 300])
def test_topology_beta_matches_the_oracle(lib, topology, n):
    from oracle import gpga_oracle as orc
    from paper_2105_09080_amd import binding as B
    for k in (0, 1, 5):
        want = orc.beta_of(orc.mixing_matrix(topology, n, k)) if n > 1 else 0.0
        # library weights are fp32 (1/3, 1/5, ...): agreement to fp32 rounding of the weights
        assert B.gpga_topology_beta(topology, n, k) == pytest.approx(want, abs=2e-7)


def test_topology_beta_large_sparse_ring(lib):
    import math
    from paper_2105_09080_amd import binding as B
    n = 1024                                                   # 1 - beta = (2/3)(1 - cos(2 pi / n))
    assert B.gpga_topology_beta("ring", n) == pytest.approx((1 + 2 * math.cos(2 * math.pi / n)) / 3, abs=2e-7)
    with pytest.raises(B.GpgaError):
        B.gpga_topology_beta("custom", 8)
    with pytest.raises(B.GpgaError):
        B.gpga_topology_beta("ring", 0)


def test_check_mixing_csr_accepts_doubly_stochastic_and_rejects_the_rest(lib):
    import numpy as np
    from oracle import gpga_oracle as orc
    from paper_2105_09080_amd import binding as B
    rng = np.random.default_rng(5)
    n = 9
    w = rng.random(4)
    w /= w.sum()
    W = w[0] * np.eye(n) + sum(w[t + 1] * np.eye(n)[rng.permutation(n)] for t in range(3))
    ptr, col, val = _dense_to_csr(W)
    W32 = np.zeros((n, n))
    W32[np.repeat(np.arange(n), np.diff(ptr)), col] = val.astype(np.float64)
    assert B.gpga_check_mixing_csr(n, ptr, col, val) == pytest.approx(orc.beta_of(W32), abs=1e-9)

    def rejected(p, c, v):
        with pytest.raises(B.GpgaError) as e:
            B.gpga_check_mixing_csr(n, p, c, v)
        return e.value.status == B.GPGA_EINVAL

    bad = val.copy(); bad[0] *= 1.01
    assert rejected(ptr, col, bad)                             # a row sum is off
    Wr = W.copy(); Wr[[0, 1]] = Wr[[1, 0]]; Wr[0] = W[0]       # row-stochastic only
    Wr[1] = W[0]
    assert rejected(*_dense_to_csr(Wr))                        # column sums are off
    neg = val.copy(); neg[0] = -neg[0]
    assert rejected(ptr, col, neg)
    oob = col.copy(); oob[2] = n
    assert rejected(ptr, oob, val)
    p2 = ptr.copy(); p2[0] = 1
    assert rejected(p2, col, val)
    p3 = ptr.copy(); p3[3], p3[4] = p3[4], p3[3] - 1
    assert rejected(p3, col, val)
    nan = val.copy(); nan[1] = float("nan")
    assert rejected(ptr, col, nan)


def test_the_header_is_plain_c_and_a_c_caller_links(tmp_path):
    """include/gpga.h compiled as C99 (pedantic, warnings are errors) from a caller that walks through
    the basic sequence of calls, linked against the built library (nothing runs: no GPU here)."""
    import shutil
    import subprocess
    from paper_2105_09080_amd import build as gbuild
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "caller.c"
    src.write_text(r'''
#include <stddef.h>
#include "gpga.h"
int run(float* x, float* xn, float* m, float* g, int32_t n, int64_t d, void* stream, double* out) {
    gpga_ctx* ctx = NULL;
    float* live = NULL;
    int64_t k;
    if (gpga_create(&ctx, n, d, GPGA_TOPO_EXPO1, 6, 1e-4f, 0.9f) != GPGA_OK) return 1;
    if (gpga_bind(ctx, x, xn, m, g, d, stream) != GPGA_OK) return 2;
    if (gpga_problem_synthetic(ctx, 0u, 1e-3f) != GPGA_OK) return 3;
    if (gpga_reset(ctx, NULL) != GPGA_OK) return 4;
    for (k = 0; k < 12; ++k) {
        if (gpga_local_grad(ctx, NULL, 0) != GPGA_OK) return 5;
        if (gpga_step(ctx) != GPGA_OK) return 6;
    }
    if (gpga_current_x(ctx, &live) != GPGA_OK || live == NULL) return 7;
    if (gpga_consensus_error(ctx, out) != GPGA_OK) return 8;
    return gpga_destroy(ctx) == GPGA_OK ? 0 : 9;
}
int main(void) { return gpga_version() == NULL; }
''')
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    obj = tmp_path / "caller.o"
    res = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                          "-c", str(src), "-o", str(obj)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    if not os.path.exists(gbuild.LIB_PATH):
        pytest.skip("library not built")
    res = subprocess.run([gcc, str(obj), "-o", str(tmp_path / "caller"), gbuild.LIB_PATH,
                          "-Wl,--unresolved-symbols=ignore-in-shared-libs"], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
