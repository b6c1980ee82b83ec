"""Driver for the transient-stage study of the paper's logistic-regression
simulation (Sec. 5.1, App. F.2): Parallel SGD, Gossip SGD, Local SGD and
Gossip-PGA on the same data, same minibatches and the same halving step-size
rule, over ring / grid / exponential graphs.

This module only sequences calls of the C ABI and collects what they produce;
gradients, updates, mixing, averaging, losses and the consensus trace are all
computed by libgpga's kernels.  Data follow the recipe the paper states (sizes,
distributions), regenerated from seeds; nothing of the paper's own data is used.

    python -m paper_2105_09080_amd.transient --n 20 50 100 --trials 3 --iters 3000
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np
import torch

from . import binding as B
from . import inputs
from .harness import Simulation

#: method -> (topology override or None, averaging period as a function of H)
METHODS = {
    "parallel": ("full", lambda H: 0),      # W = (1/n) 1 1^T : global average every iteration (Sec. 3)
    "gossip": (None, lambda H: 0),          # H -> infinity
    "local": ("none", lambda H: H),         # W = I
    "pga": (None, lambda H: H),
}


class LossProbe:
    """f(xbar) = (1/n) sum_i f_i(xbar) over each node's full local data, evaluated by the
    library on a second context whose rows are all set to xbar.  A probe only enqueues
    work (mean, row fill, loss kernels) on the simulation's stream and keeps the n losses
    on the device; ``values`` waits once and returns every f(xbar) recorded so far."""

    def __init__(self, n, d, feat_dev, y_dev, M, stream, capacity):
        self.sim = Simulation(n, d, topology="none", H=0, lr=0.0, momentum=0.0, stream=stream)
        B.gpga_problem_logreg(self.sim.ctx, feat_dev, y_dev, M)
        with torch.cuda.stream(stream):
            self.xbar = torch.empty(d, dtype=torch.float32, device=self.sim.device)
            self.losses = torch.empty(n, dtype=torch.float32, device=self.sim.device)
            self.means = torch.empty(capacity, dtype=torch.float64, device=self.sim.device)
        self.count = 0

    def __call__(self, run: Simulation):
        B.gpga_mean(run.ctx, self.xbar)
        B.gpga_reset(self.sim.ctx, self.xbar)
        B.gpga_local_loss(self.sim.ctx, None, 0, self.losses)
        B.gpga_node_mean(self.sim.ctx, self.losses, self.means[self.count:])   # f(xbar) = (1/n) sum_i f_i(xbar)
        self.count += 1

    def values(self) -> np.ndarray:
        self.sim.stream.synchronize()        # the kernels ran on the simulation's stream, not torch's current one
        return self.means[: self.count].cpu().numpy()

    def close(self):
        self.sim.close()


def run_method(method: str, topology: str, n: int, d: int, feat, y, idx, *, H: int = 16, lr0: float = 0.2,
               halve_every: int = 1000, eval_every: int = 50, momentum: float = 0.0, stream=None):
    """One trajectory.  ``idx``: (T, n, B) int32 minibatch table.  Returns a dict with the
    consensus distance after every iteration, f(xbar) every ``eval_every`` iterations and
    the iteration rate."""
    topo_override, period = METHODS[method]
    T, M = idx.shape[0], feat.shape[1]
    stream = stream or torch.cuda.Stream()
    sim = Simulation(n, d, topology=topo_override or topology, H=period(H), lr=lr0, momentum=momentum,
                     stream=stream)
    B.gpga_lr_schedule_step(sim.ctx, float(np.float32(lr0)), halve_every, 0.5)
    feat_dev, y_dev = sim.problem_logreg(feat, y)
    idx_dev = sim.upload_batches(idx)
    probe = LossProbe(n, d, feat_dev, y_dev, M, stream, capacity=T // eval_every + 2)
    trace = sim.attach_trace(T)
    probe(sim)
    at = [0]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        k = 0
        while k < T:
            chunk = min(eval_every, T - k)
            sim.run(chunk, idx_dev[k:k + chunk])          # the loop of Algorithm 1, enqueued by one call
            k += chunk
            if k % eval_every == 0:
                probe(sim)
                at.append(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    losses = probe.values()
    out = {"method": method, "topology": topo_override or topology, "n": n, "H": period(H), "iters": T,
           "iters_per_s": T / dt, "beta": sim.beta, "consensus": trace.cpu().numpy().copy(),
           "loss_at": np.asarray(at), "loss": np.asarray(losses), "x_final": sim.X.cpu().numpy()}
    probe.close()
    sim.close()
    return out


def study(ns, topology, trials, iters, *, d=10, M=8000, batch=1, H=16, iid=False, eval_every=50, seed=0,
          methods=("parallel", "gossip", "pga")):
    """Mean and standard deviation over trials of f(xbar) and of the consensus distance."""
    rows = []
    for n in ns:
        curves = {m: {"loss": [], "cons": [], "rate": []} for m in methods}
        beta = None
        for t in range(trials):
            feat, y, _ = inputs.logreg_simulation_problem(n, d, M, seed=seed + 1000 * t, iid=iid)
            idx = inputs.batch_indices(iters, n, batch, M, seed=seed + 1000 * t)
            for m in methods:
                r = run_method(m, topology, n, d, feat, y, idx, H=H, eval_every=eval_every)
                curves[m]["loss"].append(r["loss"])
                curves[m]["cons"].append(r["consensus"])
                curves[m]["rate"].append(r["iters_per_s"])
                if m == "gossip":
                    beta = r["beta"]
        for m in methods:
            L, C = np.stack(curves[m]["loss"]), np.stack(curves[m]["cons"])
            rows.append({"n": n, "topology": topology, "method": m, "beta": beta, "trials": trials,
                         "iters": iters, "loss_final_mean": float(L[:, -1].mean()),
                         "loss_final_std": float(L[:, -1].std()),
                         "loss_curve_mean": [float(v) for v in L.mean(axis=0)],
                         "consensus_mean_last_period": float(C[:, -H:].mean()),
                         "iters_per_s": float(np.mean(curves[m]["rate"]))})
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--n", type=int, nargs="+", default=[20, 50, 100])
    ap.add_argument("--topology", default="ring", choices=["ring", "grid", "expo", "expo1"])
    ap.add_argument("--trials", type=int, default=3)
    ap.add_argument("--iters", type=int, default=3000)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--H", type=int, default=16)
    ap.add_argument("--iid", action="store_true")
    ap.add_argument("--methods", nargs="+", default=["parallel", "gossip", "pga"], choices=sorted(METHODS))
    args = ap.parse_args()
    rows = study(args.n, args.topology, args.trials, args.iters, batch=args.batch, H=args.H, iid=args.iid,
                 methods=tuple(args.methods))
    for r in rows:
        r = dict(r)
        curve = r.pop("loss_curve_mean")
        r["loss_curve_mean_every_10th"] = curve[::10]
        print(json.dumps(r))


if __name__ == "__main__":
    main()
