"""ctypes binding of libgpga.so: one Python function per C entry point, same names.

Argument marshalling only - every step of the method runs in the HIP kernels
behind the C ABI (include/gpga.h).  Device arrays are passed as torch tensors
(their ``data_ptr()``) or as raw integer addresses; PyTorch is used for device
memory and streams, nothing else.  There is no CPU fallback: if the shared
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libgpga.so")

GPGA_OK, GPGA_EINVAL, GPGA_ENOMEM, GPGA_EDEVICE, GPGA_ESTATE = 0, 1, 2, 3, 4
GPGA_TOPO_RING, GPGA_TOPO_EXPO1, GPGA_TOPO_NONE, GPGA_TOPO_FULL = 0, 1, 2, 3
GPGA_TOPO_GRID, GPGA_TOPO_EXPO, GPGA_TOPO_CUSTOM = 4, 5, 6
TOPOLOGY = {"ring": GPGA_TOPO_RING, "expo1": GPGA_TOPO_EXPO1, "none": GPGA_TOPO_NONE,
            "full": GPGA_TOPO_FULL, "grid": GPGA_TOPO_GRID, "expo": GPGA_TOPO_EXPO,
            "custom": GPGA_TOPO_CUSTOM}
_STATUS_NAME = {0: "GPGA_OK", 1: "GPGA_EINVAL", 2: "GPGA_ENOMEM", 3: "GPGA_EDEVICE", 4: "GPGA_ESTATE"}

#: every symbol include/gpga.h declares: (name, restype, argtypes)
_c = ctypes
_ctx_p = _c.c_void_p
SIGNATURES = [
    ("gpga_create", _c.c_int, [_c.POINTER(_ctx_p), _c.c_int32, _c.c_int64, _c.c_int32, _c.c_int64,
                               _c.c_float, _c.c_float]),
    ("gpga_destroy", _c.c_int, [_ctx_p]),
    ("gpga_bind", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int64,
                             _c.c_void_p]),
    ("gpga_reset", _c.c_int, [_ctx_p, _c.c_void_p]),
    ("gpga_set_lr", _c.c_int, [_ctx_p, _c.c_float]),
    ("gpga_set_period", _c.c_int, [_ctx_p, _c.c_int64]),
    ("gpga_set_nesterov", _c.c_int, [_ctx_p, _c.c_int32]),
    ("gpga_lr_schedule_step", _c.c_int, [_ctx_p, _c.c_float, _c.c_int64, _c.c_float]),
    ("gpga_lr_schedule_milestones", _c.c_int, [_ctx_p, _c.c_float, _c.c_int64, _c.c_float,
                                               _c.POINTER(_c.c_int64), _c.c_int32, _c.c_float]),
    ("gpga_lr_schedule_poly", _c.c_int, [_ctx_p, _c.c_float, _c.c_int64, _c.c_int64, _c.c_float]),
    ("gpga_lr", _c.c_float, [_ctx_p]),
    ("gpga_set_iter", _c.c_int, [_ctx_p, _c.c_int64]),
    ("gpga_iter", _c.c_int64, [_ctx_p]),
    ("gpga_problem_lsq", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_void_p, _c.c_int32]),
    ("gpga_problem_logreg", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_void_p, _c.c_int32]),
    ("gpga_problem_logreg_virtual", _c.c_int, [_ctx_p, _c.c_uint64, _c.c_void_p, _c.c_int32, _c.c_float]),
    ("gpga_problem_synthetic", _c.c_int, [_ctx_p, _c.c_uint64, _c.c_float]),
    ("gpga_local_grad", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_int32]),
    ("gpga_local_loss", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_int32, _c.c_void_p]),
    ("gpga_step", _c.c_int, [_ctx_p]),
    ("gpga_run", _c.c_int, [_ctx_p, _c.c_int64, _c.c_void_p, _c.c_int32]),
    ("gpga_set_mixing_csr", _c.c_int, [_ctx_p, _c.POINTER(_c.c_int64), _c.POINTER(_c.c_int32),
                                       _c.POINTER(_c.c_float)]),
    ("gpga_mixing_beta", _c.c_int, [_ctx_p, _c.POINTER(_c.c_double)]),
    ("gpga_topology_beta", _c.c_int, [_c.c_int32, _c.c_int32, _c.c_int64, _c.POINTER(_c.c_double)]),
    ("gpga_check_mixing_csr", _c.c_int, [_c.c_int32, _c.POINTER(_c.c_int64), _c.POINTER(_c.c_int32),
                                         _c.POINTER(_c.c_float), _c.POINTER(_c.c_double)]),
    ("gpga_aga_enable", _c.c_int, [_ctx_p, _c.c_int64, _c.c_int64, _c.c_int64]),
    ("gpga_aga_step", _c.c_int, [_ctx_p, _c.c_void_p]),
    ("gpga_period", _c.c_int64, [_ctx_p]),
    ("gpga_consensus_error", _c.c_int, [_ctx_p, _c.POINTER(_c.c_double)]),
    ("gpga_consensus_error_static", _c.c_int, [_ctx_p, _c.c_void_p]),
    ("gpga_set_trace", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_int64]),
    ("gpga_mean", _c.c_int, [_ctx_p, _c.c_void_p]),
    ("gpga_node_mean", _c.c_int, [_ctx_p, _c.c_void_p, _c.c_void_p]),
    ("gpga_current_x", _c.c_int, [_ctx_p, _c.POINTER(_c.c_void_p)]),
    ("gpga_set_option", _c.c_int, [_ctx_p, _c.c_char_p, _c.c_int64]),
    ("gpga_tune", _c.c_int, [_ctx_p, _c.c_int32]),
    ("gpga_query", _c.c_int, [_ctx_p, _c.c_char_p, _c.POINTER(_c.c_double)]),
    ("gpga_probe_stream", _c.c_int, [_c.c_int32, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int64,
                                     _c.c_int32, _c.c_void_p]),
    ("gpga_last_error", _c.c_char_p, [_ctx_p]),
    ("gpga_version", _c.c_char_p, []),
]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2105_09080_amd/build.py).  There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    for name, restype, argtypes in SIGNATURES:
        fn = getattr(lib, name)          # AttributeError if the library lacks a declared symbol
        fn.restype = restype
        fn.argtypes = argtypes
    return lib


_lib = _load()


class GpgaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAME.get(status, status)}: {message}")
        self.status = status


def _ptr(t):
    """Device address of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(ctx, status: int):
    if status != GPGA_OK:
        msg = _lib.gpga_last_error(ctx) if ctx else b""
        raise GpgaError(status, (msg or b"").decode())


# ---- one function per C entry point -----------------------------------------

def gpga_create(n: int, d: int, topology, H: int, lr: float, momentum: float):
    """Returns an opaque context handle (int).  ``topology``: name or enum value."""
    topo = TOPOLOGY[topology] if isinstance(topology, str) else int(topology)
    out = _ctx_p()
    status = _lib.gpga_create(ctypes.byref(out), n, d, topo, H, lr, momentum)
    if status != GPGA_OK:
        raise GpgaError(status, "gpga_create rejected its arguments" if status == GPGA_EINVAL
                        else "gpga_create failed")
    return out.value


def gpga_destroy(ctx):
    _check(None, _lib.gpga_destroy(ctx))


def gpga_bind(ctx, x, x_new, m, g, ld: int, stream=None):
    """x, x_new, m, g: torch CUDA tensors (or addresses); stream: hipStream_t address or None."""
    _check(ctx, _lib.gpga_bind(ctx, _ptr(x), _ptr(x_new), _ptr(m), _ptr(g), ld, stream))


def gpga_reset(ctx, x0=None):
    _check(ctx, _lib.gpga_reset(ctx, _ptr(x0)))


def gpga_set_lr(ctx, lr: float):
    _check(ctx, _lib.gpga_set_lr(ctx, lr))


def gpga_set_period(ctx, H: int):
    _check(ctx, _lib.gpga_set_period(ctx, H))


def gpga_set_nesterov(ctx, on: bool):
    _check(ctx, _lib.gpga_set_nesterov(ctx, int(on)))


def gpga_lr_schedule_step(ctx, base_lr: float, period: int, factor: float):
    _check(ctx, _lib.gpga_lr_schedule_step(ctx, base_lr, period, factor))


def gpga_lr_schedule_milestones(ctx, base_lr: float, warmup_iters: int, warmup_start_lr: float,
                                milestones, factor: float):
    ms = [int(v) for v in milestones]
    arr = (ctypes.c_int64 * max(1, len(ms)))(*ms)
    _check(ctx, _lib.gpga_lr_schedule_milestones(ctx, base_lr, warmup_iters, warmup_start_lr, arr,
                                                  len(ms), factor))


def gpga_lr_schedule_poly(ctx, base_lr: float, warmup_iters: int, total_iters: int, power: float):
    _check(ctx, _lib.gpga_lr_schedule_poly(ctx, base_lr, warmup_iters, total_iters, power))


def gpga_lr(ctx) -> float:
    return float(_lib.gpga_lr(ctx))


def gpga_set_iter(ctx, k: int):
    _check(ctx, _lib.gpga_set_iter(ctx, k))


def gpga_iter(ctx) -> int:
    return int(_lib.gpga_iter(ctx))


def gpga_problem_lsq(ctx, A, b, M: int):
    _check(ctx, _lib.gpga_problem_lsq(ctx, _ptr(A), _ptr(b), M))


def gpga_problem_logreg(ctx, feat, y, M: int):
    _check(ctx, _lib.gpga_problem_logreg(ctx, _ptr(feat), _ptr(y), M))


def gpga_problem_logreg_virtual(ctx, seed: int, y, M: int, mu_var: float):
    _check(ctx, _lib.gpga_problem_logreg_virtual(ctx, seed, _ptr(y), M, mu_var))


def gpga_problem_synthetic(ctx, seed: int, grad_var: float):
    _check(ctx, _lib.gpga_problem_synthetic(ctx, seed, grad_var))


def gpga_local_grad(ctx, batch_idx=None, B: int = 0):
    _check(ctx, _lib.gpga_local_grad(ctx, _ptr(batch_idx), B))


def gpga_local_loss(ctx, batch_idx, B: int, loss):
    _check(ctx, _lib.gpga_local_loss(ctx, _ptr(batch_idx), B, _ptr(loss)))


def gpga_step(ctx):
    _check(ctx, _lib.gpga_step(ctx))


def _csr_arrays(row_ptr, col, val):
    rp = [int(v) for v in row_ptr]
    cl = [int(v) for v in col]
    vl = [float(v) for v in val]
    return ((ctypes.c_int64 * len(rp))(*rp), (ctypes.c_int32 * max(1, len(cl)))(*cl),
            (ctypes.c_float * max(1, len(vl)))(*vl))


def gpga_set_mixing_csr(ctx, row_ptr, col, val):
    """row_ptr (n+1), col, val: host sequences (lists or NumPy arrays)."""
    rp, cl, vl = _csr_arrays(row_ptr, col, val)
    _check(ctx, _lib.gpga_set_mixing_csr(ctx, rp, cl, vl))


def gpga_mixing_beta(ctx) -> float:
    out = ctypes.c_double()
    _check(ctx, _lib.gpga_mixing_beta(ctx, ctypes.byref(out)))
    return out.value


def gpga_topology_beta(topology, n: int, k: int = 0) -> float:
    topo = TOPOLOGY[topology] if isinstance(topology, str) else int(topology)
    out = ctypes.c_double()
    status = _lib.gpga_topology_beta(topo, n, k, ctypes.byref(out))
    if status != GPGA_OK:
        raise GpgaError(status, "gpga_topology_beta rejected its arguments")
    return out.value


def gpga_check_mixing_csr(n: int, row_ptr, col, val) -> float:
    """Validates W; returns its beta.  Raises GpgaError(EINVAL) if W is rejected."""
    rp, cl, vl = _csr_arrays(row_ptr, col, val)
    out = ctypes.c_double()
    status = _lib.gpga_check_mixing_csr(n, rp, cl, vl, ctypes.byref(out))
    if status != GPGA_OK:
        raise GpgaError(status, "mixing matrix rejected")
    return out.value


def gpga_run(ctx, T: int, batch_table=None, B: int = 0):
    _check(ctx, _lib.gpga_run(ctx, T, _ptr(batch_table), B))


def gpga_aga_enable(ctx, H_init: int, warmup_iters: int, H_max: int):
    _check(ctx, _lib.gpga_aga_enable(ctx, H_init, warmup_iters, H_max))


def gpga_aga_step(ctx, loss):
    _check(ctx, _lib.gpga_aga_step(ctx, _ptr(loss)))


def gpga_period(ctx) -> int:
    return int(_lib.gpga_period(ctx))


def gpga_consensus_error(ctx) -> float:
    out = ctypes.c_double()
    _check(ctx, _lib.gpga_consensus_error(ctx, ctypes.byref(out)))
    return out.value


def gpga_consensus_error_static(ctx, out):
    """out: float64 CUDA tensor (or address) receiving the consensus distance; nothing is allocated."""
    _check(ctx, _lib.gpga_consensus_error_static(ctx, _ptr(out)))


def gpga_set_trace(ctx, trace, capacity: int = 0):
    """trace: float64 CUDA tensor (or address) with ``capacity`` entries; None detaches."""
    _check(ctx, _lib.gpga_set_trace(ctx, _ptr(trace), capacity))


def gpga_mean(ctx, xbar):
    _check(ctx, _lib.gpga_mean(ctx, _ptr(xbar)))


def gpga_node_mean(ctx, v, out):
    """v: n floats on the device; out: one float64 on the device."""
    _check(ctx, _lib.gpga_node_mean(ctx, _ptr(v), _ptr(out)))


def gpga_current_x(ctx) -> int:
    out = ctypes.c_void_p()
    _check(ctx, _lib.gpga_current_x(ctx, ctypes.byref(out)))
    return out.value


def gpga_set_option(ctx, name: str, value: int):
    _check(ctx, _lib.gpga_set_option(ctx, name.encode(), value))


def gpga_tune(ctx, launches: int):
    _check(ctx, _lib.gpga_tune(ctx, launches))


def gpga_query(ctx, name: str) -> float:
    out = ctypes.c_double()
    _check(ctx, _lib.gpga_query(ctx, name.encode(), ctypes.byref(out)))
    return out.value


def gpga_probe_stream(kind: int, src, dst, nbytes: int, stream=None, src2=None, inout=None, blocks_per_cu: int = 0):
    """kind 0 read src (dst: 4-byte sink), 1 write dst, 2 copy src -> dst, 3 read src, src2, inout and
    write inout, dst; enqueued on ``stream``."""
    status = _lib.gpga_probe_stream(kind, _ptr(src), _ptr(dst), _ptr(src2), _ptr(inout), nbytes, blocks_per_cu,
                                    stream)
    if status != GPGA_OK:
        raise GpgaError(status, "gpga_probe_stream rejected its arguments or failed to launch")


def gpga_last_error(ctx) -> str:
    return (_lib.gpga_last_error(ctx) or b"").decode()


def gpga_version() -> str:
    return _lib.gpga_version().decode()


def raw_status(name: str, *args) -> int:
    """Call an entry point and return its raw status (for error-path tests)."""
    return getattr(_lib, name)(*args)
