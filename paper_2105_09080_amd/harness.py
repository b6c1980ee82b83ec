"""Device-memory plumbing around the C ABI: allocates the n x d state with
PyTorch-ROCm, binds it, and keeps the tensors alive.  No arithmetic of the
method happens here - every update goes through libgpga."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class Simulation:
    """n simulated nodes with d parameters each on one GPU.

    Owns four (n, ld) fp32 CUDA tensors (x, x_new, m, g) and a libgpga context
    bound to them on ``stream`` (a torch.cuda.Stream; default: current stream).
    """

    def __init__(self, n: int, d: int, *, topology: str, H: int, lr: float, momentum: float = 0.0,
                 ld: int | None = None, device: str = "cuda:0", stream: torch.cuda.Stream | None = None,
                 x0=None, alloc_m: bool | None = None):
        if not torch.cuda.is_available():
            raise RuntimeError("libgpga needs a GPU (torch.cuda.is_available() is False)")
        self.n, self.d = n, d
        self.ld = d if ld is None else ld
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.ctx = B.gpga_create(n, d, topology, H, lr, momentum)
        with torch.cuda.stream(self.stream):
            self._bufs = [torch.empty((n, self.ld), dtype=torch.float32, device=self.device) for _ in range(2)]
            need_m = (momentum != 0.0) if alloc_m is None else alloc_m
            self.m = torch.zeros((n, self.ld), dtype=torch.float32, device=self.device) if need_m else None
            self.g = torch.zeros((n, self.ld), dtype=torch.float32, device=self.device)
        self._addr = {t.data_ptr(): t for t in self._bufs}
        B.gpga_bind(self.ctx, self._bufs[0], self._bufs[1], self.m, self.g, self.ld, self.stream.cuda_stream)
        self._keep = []
        x0_dev = None
        if x0 is not None:
            x0_dev = torch.as_tensor(np.asarray(x0, dtype=np.float32)).to(self.device)
            self._keep.append(x0_dev)
        self.stream.synchronize()
        B.gpga_reset(self.ctx, x0_dev)

    # -- state access -----------------------------------------------------------
    @property
    def X(self) -> torch.Tensor:
        """Live iterates, (n, d) view of the (n, ld) buffer."""
        return self._addr[B.gpga_current_x(self.ctx)][:, : self.d]

    @property
    def G(self) -> torch.Tensor:
        return self.g[:, : self.d]

    @property
    def M(self):
        return None if self.m is None else self.m[:, : self.d]

    @property
    def k(self) -> int:
        return B.gpga_iter(self.ctx)

    def set_state(self, X=None, M=None, G=None, k=None):
        """Overwrite device state from host arrays (lock-step comparisons)."""
        with torch.cuda.stream(self.stream):
            if X is not None:
                self.X.copy_(torch.as_tensor(np.asarray(X, dtype=np.float32)))
            if M is not None and self.m is not None:
                self.M.copy_(torch.as_tensor(np.asarray(M, dtype=np.float32)))
            if G is not None:
                self.G.copy_(torch.as_tensor(np.asarray(G, dtype=np.float32)))
        self.stream.synchronize()
        if k is not None:
            B.gpga_set_iter(self.ctx, k)

    # -- problems ------------------------------------------------------------------
    def _upload(self, a, dtype):
        t = torch.as_tensor(np.ascontiguousarray(a)).to(dtype).to(self.device)
        self._keep.append(t)
        return t

    def problem_lsq(self, A, b):
        A_d, b_d = self._upload(A, torch.float32), self._upload(b, torch.float32)
        B.gpga_problem_lsq(self.ctx, A_d, b_d, A.shape[1])
        return A_d, b_d

    def problem_logreg(self, feat, y):
        f_d, y_d = self._upload(feat, torch.float32), self._upload(y, torch.float32)
        B.gpga_problem_logreg(self.ctx, f_d, y_d, feat.shape[1])
        return f_d, y_d

    def problem_logreg_virtual(self, seed: int, y, mu_var: float):
        y_d = self._upload(y, torch.float32)
        B.gpga_problem_logreg_virtual(self.ctx, seed, y_d, y.shape[1], mu_var)
        return y_d

    def problem_synthetic(self, seed: int, grad_var: float):
        B.gpga_problem_synthetic(self.ctx, seed, grad_var)

    def upload_batches(self, idx):
        """(T, n, B) int32 minibatch table -> device tensor."""
        return self._upload(idx, torch.int32)

    # -- the iteration -------------------------------------------------------------
    def local_grad(self, batch_idx=None):
        if batch_idx is None:
            B.gpga_local_grad(self.ctx, None, 0)
        else:
            B.gpga_local_grad(self.ctx, batch_idx, batch_idx.shape[-1])

    def local_loss(self, batch_idx=None) -> torch.Tensor:
        out = torch.empty(self.n, dtype=torch.float32, device=self.device)
        B.gpga_local_loss(self.ctx, batch_idx, 0 if batch_idx is None else batch_idx.shape[-1], out)
        return out

    def step(self):
        B.gpga_step(self.ctx)

    def set_mixing(self, W):
        """Attach a dense (n, n) doubly stochastic W: its non-zeros are handed over in CSR form."""
        W = np.asarray(W)
        rows, cols = np.nonzero(W)          # row-major order
        ptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=self.n))])
        B.gpga_set_mixing_csr(self.ctx, ptr, cols, W[rows, cols].astype(np.float32))

    @property
    def beta(self) -> float:
        return B.gpga_mixing_beta(self.ctx)

    def set_nesterov(self, on: bool = True):
        B.gpga_set_nesterov(self.ctx, on)

    @property
    def lr(self) -> float:
        """Step size the next step will use."""
        return B.gpga_lr(self.ctx)

    def run(self, T: int, batch_table=None):
        """T iterations (gradient + step) from one call; batch_table: (>= T, n, B) int32 device tensor."""
        if batch_table is None:
            B.gpga_run(self.ctx, T, None, 0)
        else:
            assert batch_table.shape[0] >= T and batch_table.is_contiguous()
            B.gpga_run(self.ctx, T, batch_table, batch_table.shape[-1])

    def aga_enable(self, H_init: int, warmup_iters: int, H_max: int):
        B.gpga_aga_enable(self.ctx, H_init, warmup_iters, H_max)

    def aga_step(self, loss: torch.Tensor):
        B.gpga_aga_step(self.ctx, loss)

    @property
    def period(self) -> int:
        return B.gpga_period(self.ctx)

    def consensus_error(self) -> float:
        return B.gpga_consensus_error(self.ctx)

    def consensus_error_static(self, out: torch.Tensor):
        """Consensus distance into ``out`` (one float64 on the device), asynchronously, no allocation."""
        B.gpga_consensus_error_static(self.ctx, out)

    def attach_trace(self, capacity: int) -> torch.Tensor:
        """Device array that receives the consensus distance after every step (no host sync)."""
        self.trace = torch.full((capacity,), float("nan"), dtype=torch.float64, device=self.device)
        self.stream.synchronize()
        B.gpga_set_trace(self.ctx, self.trace, capacity)
        return self.trace

    def mean(self) -> torch.Tensor:
        out = torch.empty(self.d, dtype=torch.float32, device=self.device)
        B.gpga_mean(self.ctx, out)
        return out

    def tune(self, launches: int = 16):
        """Let the pacing controllers settle (state arrays are left with unspecified contents)."""
        B.gpga_tune(self.ctx, launches)

    def query(self, name: str) -> float:
        return B.gpga_query(self.ctx, name)

    def set_option(self, name: str, value: int):
        B.gpga_set_option(self.ctx, name, value)

    def close(self):
        if self.ctx is not None:
            B.gpga_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
