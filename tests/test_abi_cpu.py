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
    assert call(topo=4) == B.GPGA_EINVAL
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
