#!/usr/bin/env python3
"""Benchmark of the Gossip-PGA hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
gpga_local_grad (counter-RNG gradients written to the resident G buffer) followed
by gpga_step (fused momentum + local update + gossip mix, or the exact all-node
mean every H-th step).  All buffers (x, x_new, m, g) are resident in HBM before
the timed region starts.

Prints ONE JSON line.  `value` is steps/s of the whole path on the primary
workload (cfg3: n=64, d=25.6M, the ResNet-50-sized configuration); the
`roofline` object is for the dominant kernel (the fused gossip step), timed
live with HIP events on the stream the kernels are launched on; `cpu_baseline`
is the NumPy oracle timed on a bounded column slab of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
BYTES_PER_ELT = 20             # read x, m, g; write m, x_new (fp32)

# HBM bytes per launch of the fused gossip step measured with rocprofv3 --pmc
# (FETCH_SIZE run + WRITE_SIZE run, scaled by a copy kernel of known size); the
# summaries live under profiles/.  None = not measured for that workload.
# These are constants copied from those summaries, NOT something a bench run measures: the JSON line
# carries them as `traffic` together with `traffic_source`.
MEASURED_TRAFFIC_BYTES = {
    # 12.000 B fetched + 8.000 B written per element in every case; where several kernels share the gossip steps
    # (one per one-peer offset class) the largest of their per-launch figures is given
    "cfg3/ring": (32768427004, "profiles/step_cfg3_ring.md"),          # k_step_walk
    "cfg3/expo1": (32768515517, "profiles/step_cfg3_expo1.md"),        # k_step_walk (offsets 1, 2), k_step_cycles (4 .. 32)
    "cfg4/expo1": (140800368980, "profiles/step_cfg4_expo1.md"),       # k_step_walk (offset 1), k_step_cycles (2 .. 16)
    "cfg5/ring": (20480467145, "profiles/step_cfg5_ring.md"),          # k_step_walk with the consensus trace riding along
    "cfg3/grid": (32768670746, "profiles/step_sparse_cfg3_grid.md"),   # k_step_tile
    "cfg5/grid": (20480767643, "profiles/step_sparse_cfg5_grid.md"),   # k_step_band with the consensus trace riding along
}


# The paper's own wall-clock figures (its appendix on communication overhead: mean iteration time in
# ms over 500 iterations, communication part in the paper's parentheses = total - no-communication).
# Whole-cluster numbers on other hardware: context for the reader, never a baseline for this metric.
PAPER_CONTEXT = {
    "source": "arXiv 2105.09080, appendix comparing gossip and All-Reduce overhead; set-up in App. F.1",
    "hardware": "servers of 8 x V100, PyTorch 1.5.1 + NCCL 2.5.7, 25 Gbps TCP between servers, mixed precision",
    "iteration_ms": {
        "ResNet-50 (~25.5M parameters), 32 servers": {"no_communication": 146, "all_reduce": 424, "gossip": 296},
        "BERT-Large, 8 servers": {"no_communication": 445, "all_reduce": 1913.8, "gossip": 1011.5},
    },
    "note": "on one MI355X the gossip exchange and the all-reduce are HBM traffic of the fused step: "
            "5.3 ms (25.6M parameters, 64 simulated nodes) against the paper's 150 ms / 278 ms of network time",
}


# gpga_query "step_path" -> kernel
PATH_NAMES = {1: "k_step_walk", 2: "k_step_cycles", 3: "k_step_global", 4: "k_step_tile", 5: "k_step_band",
              6: "W = I walk + k_spmm_rows", 7: "k_small_run"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg3",
                    help="primary workload: cfg3 (default) or cfg4 for the bandwidth figure; cfg5, and the small cfg1 / cfg2 "
                         "(launch-latency bound: their roofline block is context only), for profiles")
    ap.add_argument("--topology", default=None,
                    help="ring, expo1, grid, expo, none or full (default: first listed for the workload)")
    ap.add_argument("--also", default="cfg3:expo1,cfg4:expo1,cfg5:ring",
                    help="comma list of extra workload:topology pairs measured after the primary ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small", action="store_true",
                    help="skip the iterations/s measurement on the shape of the paper's logistic simulation")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="run this many plain device copies of one n x d buffer before the timed loop "
                         "(a kernel of known size: reads and writes 4*n*d bytes; used to scale rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--trace", type=int, default=-1,
                    help="1 = record the consensus distance after every step on the device (gpga_set_trace), "
                         "0 = do not; default: on for cfg5 (which reports it), off otherwise")
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark, measure the chip's plain read / write / copy rates with the "
                         "library's streaming probe and the W = I fused step (3 reads : 2 writes, no mixing) on "
                         "the cfg3 shape; prints one JSON line")
    ap.add_argument("--cfg5-sweep", type=int, default=0, metavar="T",
                    help="instead of the benchmark, run cfg5 (n=1024, d=1M, virtual-feature logistic regression) "
                         "for T steps over ring and one-peer topologies and H in {1, 8, 64, never}, recording the "
                         "consensus distance after every step on the device; prints one JSON line per run")
    ap.add_argument("--opt", action="append", default=[], help="launch option name=value (repeatable)")
    return ap.parse_args()


def window_start(H, T, steps):
    """First iteration of the timed window.  A run of at least H steps (or a workload that never
    averages) starts at iteration 0 as the workload states.  A shorter run times the LAST `steps`
    iterations of the first averaging period, steps H - steps .. H - 1, so that the window ends with
    a global-average step and (for windows of at least 8 steps of the one-peer graph with 6 offsets)
    still holds every offset: the offset whose turn coincides with the averaging step shows up one
    cycle of offsets earlier."""
    if H <= 0 or steps >= H:
        return 0
    return H - steps


def one_peer_offset(n, k):
    tau = max(1, (n - 1).bit_length())
    return (1 << (k % tau)) % n


def run_workload(cfg_name, topology, steps, warmup, opts, copy_probe=0, trace=-1):
    """Times `steps` passes of local_grad + step.  Returns a dict of measurements."""
    import torch

    from paper_2105_09080_amd import binding as B
    from paper_2105_09080_amd import inputs
    from paper_2105_09080_amd.harness import Simulation

    c = inputs.CONFIGS[cfg_name]
    n, d = c["n"], c["d"]
    stream = torch.cuda.Stream()
    sim = Simulation(n, d, topology=topology, H=c["H"], lr=c["lr"], momentum=c["momentum"], stream=stream)
    for name, v in opts.items():
        sim.set_option(name, v)
    if c["problem"] == "synthetic":
        sim.problem_synthetic(c["seed"], c["grad_var"])
        grad = sim.local_grad
    elif c["problem"] == "lsq":  # cfg1: stored least-squares blocks, full batch
        A, b, _ = inputs.lsq_problem(n, d, c["M"], c["seed"], c["noise_std"])
        sim.problem_lsq(A, b)
        grad = sim.local_grad
    elif c["problem"] == "logreg":  # cfg2: stored logistic-regression features, minibatches drawn by the caller
        feat, y, _ = inputs.logreg_problem(n, d, c["M"], c["seed"], c["mu_var"], c["label_noise_std"])
        sim.problem_logreg(feat, y)
        idx = sim.upload_batches(inputs.batch_indices(max(c["H"], 0) + steps + warmup, n, c["B"], c["M"], c["seed"]))
        grad = lambda: sim.local_grad(idx[sim.k])
    else:  # cfg5: virtual-feature logistic regression
        y = inputs.virtual_labels(n, c["M"], c["seed"])
        sim.problem_logreg_virtual(c["seed"], y, c["mu_var"])
        idx = sim.upload_batches(inputs.batch_indices(max(c["H"], 0) + steps + warmup, n, c["B"], c["M"], c["seed"]))
        grad = lambda: sim.local_grad(idx[sim.k])

    want_trace = (cfg_name == "cfg5") if trace < 0 else bool(trace)
    k_first = window_start(c["H"], c["T"], steps)
    k_warm = max(0, k_first - warmup)
    trace_dev = sim.attach_trace(k_first + steps + warmup) if want_trace else None
    with torch.cuda.stream(stream):
        for _ in range(copy_probe):
            sim._bufs[1].copy_(sim._bufs[0])
        # persistent launches find their pacing rate by themselves, a dozen launches per kind of step:
        # let that happen before the W warm-up steps, then start again from x0 = 0
        sim.tune(32)
        B.gpga_reset(sim.ctx, None)
        # the iteration counter (which drives the averaging schedule, the one-peer offset and the address
        # of the synthetic gradients) is placed like on a resume: warm-up iterations lead up to the window
        sim.set_state(k=k_warm)
        for _ in range(warmup):
            grad()
            sim.step()
        sim.set_state(k=k_first)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        kinds, offsets, paths = [], [], []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            k = sim.k
            kinds.append("global" if (c["H"] > 0 and (k + 1) % c["H"] == 0) else "gossip")
            offsets.append(one_peer_offset(n, k) if topology == "expo1" else None)
            ev[i][0].record()
            grad()
            ev[i][1].record()
            sim.step()
            ev[i][2].record()
            paths.append((int(sim.query("step_path")), int(sim.query("step_paced"))))   # host-side facts, no synchronisation
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    grad_ms = [ev[i][0].elapsed_time(ev[i][1]) for i in range(steps)]
    step_ms = [ev[i][1].elapsed_time(ev[i][2]) for i in range(steps)]
    gossip = [t for t, kd in zip(step_ms, kinds) if kd == "gossip"]
    glob = [t for t, kd in zip(step_ms, kinds) if kd == "global"]
    elts = n * d
    per_offset = {}
    for t, kd, off in zip(step_ms, kinds, offsets):
        if kd == "gossip" and off is not None:
            per_offset.setdefault(off, []).append(t)
    res = {
        "workload": f"{cfg_name}: n={n} d={d} {topology} H={c['H']} momentum={c['momentum']}",
        "cfg": cfg_name, "iterations": [k_first, k_first + steps - 1],
        "gossip_ms_by_offset": {str(o): sum(v) / len(v) for o, v in sorted(per_offset.items())} or None,
        "n": n, "d": d, "topology": topology, "H": c["H"],
        "wall_s": t1 - t0,
        "ms_per_step": 1e3 * (t1 - t0) / steps,
        "steps_per_s": steps / (t1 - t0),
        "grad_ms_avg": sum(grad_ms) / steps,
        "step_ms_avg": sum(step_ms) / steps,
        "gossip_ms_avg": sum(gossip) / len(gossip) if gossip else None,
        "global_ms_avg": sum(glob) / len(glob) if glob else None,
        "n_gossip": len(gossip), "n_global": len(glob), "step_ms_each": step_ms,
        "algorithmic_bytes_per_launch": BYTES_PER_ELT * elts,
    }
    dom = res["gossip_ms_avg"] if gossip else res["global_ms_avg"]
    res["dominant"] = "gossip" if gossip else "global"
    # which kernels the gossip steps of the timed window ran as, as the library reports it
    seen = sorted({p for p, kd in zip(paths, kinds) if kd == "gossip"})
    res["gossip_kernels"] = [PATH_NAMES.get(p, str(p)) + (" (paced persistent launch)" if paced else "") for p, paced in seen]
    res["achieved_gbs"] = BYTES_PER_ELT * elts / (dom * 1e-3) / 1e9
    if glob:
        res["global_gbs"] = BYTES_PER_ELT * elts / (res["global_ms_avg"] * 1e-3) / 1e9
    res["grad_write_gbs"] = 4 * elts / (res["grad_ms_avg"] * 1e-3) / 1e9
    res["step_only_steps_per_s"] = 1e3 / res["step_ms_avg"]
    res["consensus_error_final"] = sim.consensus_error()
    # where the pacing controllers of the persistent launches ended up (device-side state, read back once)
    res["pace_controllers"] = {}
    for kind in [k + d for k in ("ring", "global", "peer_long", "peer_16", "peer_8", "peer_4", "cycles", "tile", "band", "self") for d in ("", "/1")]:
        launches = sim.query(f"pace_launches:{kind}")
        if launches > 0:
            res["pace_controllers"][kind] = {
                "rate_gbs": round(sim.query(f"pace_rate_gbs:{kind}")), "launches": int(launches),
                "late_launches": int(sim.query(f"pace_late_launches:{kind}")),
                "last_late_us": round(sim.query(f"pace_last_late_us:{kind}"), 1),
                "last_plan_us": round(sim.query(f"pace_last_plan_us:{kind}"), 1)}
    if trace_dev is not None:
        tr = trace_dev.cpu().numpy()
        tr = tr[tr == tr]          # entries of the iterations that ran (the rest is still NaN)
        res["consensus_trace"] = {"steps": int(len(tr)), "first": [float(v) for v in tr[:10]],
                                  "last": float(tr[-1]), "max": float(tr.max())}
    sim.close()
    del sim
    torch.cuda.empty_cache()
    return res


def run_probe(reps=12):
    """Machine ceilings: bytes moved / median launch time for the streaming probe kernels."""
    import torch

    from paper_2105_09080_amd import binding as B
    from paper_2105_09080_amd import inputs
    from paper_2105_09080_amd.harness import Simulation

    nbytes = 6 << 30
    stream = torch.cuda.Stream()
    out = {}
    with torch.cuda.stream(stream):
        a, b, c2, m = (torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda") for _ in range(4))
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        cases = ((0, "read_only", nbytes), (1, "write_only", nbytes), (2, "copy_1r1w", 2 * nbytes),
                 (3, "elementwise_3r2w", 5 * nbytes))
        for bpc, tag in ((0, "one_lane_per_word"), (8, "grid_stride_8_per_cu")):
            for kind, name, moved in cases:
                dst = sink if kind == 0 else b
                call = lambda: B.gpga_probe_stream(kind, a, dst, nbytes, stream.cuda_stream, src2=c2, inout=m,
                                                   blocks_per_cu=bpc)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
                call()
                ev[0].record()
                for i in range(reps):
                    call()
                    ev[i + 1].record()
                torch.cuda.synchronize()
                ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
                out[f"{name}/{tag}"] = {"gbs_median": moved / ms[len(ms) // 2] / 1e6, "gbs_best": moved / ms[0] / 1e6,
                                        "bytes": moved}
    del a, b, c2, m
    torch.cuda.empty_cache()
    c = inputs.CONFIGS["cfg3"]
    n, d = c["n"], c["d"]
    sim = Simulation(n, d, topology="none", H=0, lr=c["lr"], momentum=c["momentum"], stream=stream)
    sim.problem_synthetic(c["seed"], c["grad_var"])
    with torch.cuda.stream(stream):
        sim.local_grad()
        for _ in range(3):
            sim.step()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            sim.step()
            ev[i + 1].record()
        torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    out["fused_step_W_identity_3r2w"] = {"gbs_median": BYTES_PER_ELT * n * d / ms[len(ms) // 2] / 1e6,
                                         "gbs_best": BYTES_PER_ELT * n * d / ms[0] / 1e6,
                                         "bytes": BYTES_PER_ELT * n * d}
    sim.close()
    return {"probe": "MI355X streaming rates, 128-bit non-temporal accesses", "peak_gbs": HBM_PEAK_GBS, **out}


def run_cfg5_sweep(T):
    """cfg5 as stated: both topologies, H in {1, 8, 64, infinity}, consensus distance per step + throughput."""
    import torch

    from paper_2105_09080_amd import binding as B
    from paper_2105_09080_amd import inputs
    from paper_2105_09080_amd.harness import Simulation

    c = inputs.CONFIGS["cfg5"]
    n, d = c["n"], c["d"]
    y = inputs.virtual_labels(n, c["M"], c["seed"])
    idx_host = inputs.batch_indices(T, n, c["B"], c["M"], c["seed"])
    for topology in c["topologies"]:
        for H in c["H_sweep"]:
            stream = torch.cuda.Stream()
            sim = Simulation(n, d, topology=topology, H=H, lr=c["lr"], momentum=c["momentum"], stream=stream)
            sim.problem_logreg_virtual(c["seed"], y, c["mu_var"])
            idx = sim.upload_batches(idx_host)
            trace = sim.attach_trace(T)
            with torch.cuda.stream(stream):
                sim.run(5, idx)                     # warm-up, then start again from x0 = 0
            B.gpga_reset(sim.ctx, None)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with torch.cuda.stream(stream):
                sim.run(T, idx)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            tr = trace.cpu().numpy()
            avg_steps = [k for k in range(T) if H > 0 and (k + 1) % H == 0]
            other = [k for k in range(T) if k not in set(avg_steps)]
            print(json.dumps({
                "workload": f"cfg5: n={n} d={d} {topology} H={'inf' if H == 0 else H} T={T}",
                "steps_per_s": T / dt, "ms_per_step": 1e3 * dt / T, "node_updates_per_s": n * T / dt,
                "consensus_zero_after_every_average": bool(all(tr[k] == 0.0 for k in avg_steps)),
                "consensus_max": float(tr.max()),
                "consensus_mean_between_averages": float(tr[other].mean()) if other else 0.0,
                "consensus_last_10": [float(v) for v in tr[-10:]],
                "consensus_every_50th": [float(v) for v in tr[49::50]],
            }), flush=True)
            sim.close()
            del sim
            torch.cuda.empty_cache()


def run_simulation_shape(T=4000):
    """Iterations/s of the whole loop (gpga_run) on the shape of the paper's logistic simulation
    (Sec. 5.1: n = 100 nodes, d = 10, one sample per node and iteration, ring, H = 16, consensus
    trace on), with whole iterations in one workgroup and with one kernel per stage."""
    import torch

    from paper_2105_09080_amd import harness, inputs
    n, d, M, B = 100, 10, 8000, 1
    feat, y, _ = inputs.logreg_simulation_problem(n, d, M, seed=0)
    idx = inputs.batch_indices(T, n, B, M, seed=0)
    out = {"workload": f"Sec. 5.1 simulation shape: n={n} d={d} M={M} B={B} ring H=16, trace on", "iterations": T}
    for key, small in (("single_workgroup_iters_per_s", 1), ("kernel_per_stage_iters_per_s", 0)):
        sim = harness.Simulation(n, d, topology="ring", H=16, lr=0.2, momentum=0.0)
        sim.set_option("small_run", small)
        sim.problem_logreg(feat, y)
        idx_d = sim.upload_batches(idx)
        sim.attach_trace(2 * T)
        sim.run(T, idx_d)
        torch.cuda.synchronize()
        sim.set_state(k=0)
        t0 = time.perf_counter()
        sim.run(T, idx_d)
        torch.cuda.synchronize()
        out[key] = T / (time.perf_counter() - t0)
        sim.close()
    return out


def cpu_baseline(cfg_name, topology, budget_s=16.0):
    """The oracle as it stands on a column slab of the workload (the recursion is column-separable
    with synthetic gradients), scaled to the full width.  Two legs of about budget_s / 2 each: the
    whole path (the oracle's counter-RNG gradients + its step), which is what `value` measures on
    the GPU, and the step alone on prescribed gradients.  `cores` is what the timed code really kept
    busy: process CPU time / wall time (NumPy's elementwise work and the oracle's generator run on
    one thread, only the W @ Y product uses the BLAS pool)."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import gpga_oracle as orc
    from paper_2105_09080_amd import inputs

    c = inputs.CONFIGS[cfg_name]
    n, d = c["n"], c["d"]
    slab = 65536
    cols = np.arange(slab)
    kw = dict(topology=topology, H=c["H"], lr=c["lr"], momentum=c["momentum"], storage="f32")

    def timed(make_grad):
        ref = orc.GossipPGA(n, slab, **kw)
        w0, p0, steps = time.perf_counter(), time.process_time(), 0
        while True:
            ref.step(make_grad(steps))
            steps += 1
            if time.perf_counter() - w0 > budget_s / 2 or steps >= c["T"]:
                break
        wall, cpu = time.perf_counter() - w0, time.process_time() - p0
        return steps, wall / steps, cpu / wall

    steps_a, dt_a, busy_a = timed(lambda k: orc.synthetic_grad(c["seed"], k, n, cols, c["grad_var"]))
    G_fixed = orc.synthetic_grad(c["seed"], 0, n, cols, c["grad_var"])
    steps_b, dt_b, busy_b = timed(lambda k: G_fixed)
    blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    scale = d / slab
    return {
        "value": 1.0 / (dt_a * scale), "unit": "steps/s", "cores": max(1, round(busy_a)), "kind": "oracle",
        "step_only_value": 1.0 / (dt_b * scale), "step_only_cores": max(1, round(busy_b)),
        "busy_threads_measured": {"whole_path": busy_a, "step_only": busy_b},
        "blas_pool_threads": blas, "host_cpus": os.cpu_count(),
        "sample": f"NumPy float64 oracle on a {n}x{slab} column slab of {cfg_name}/{topology}, scaled by d/slab = {scale:.1f} "
                  f"(columns are independent): whole path (counter-RNG gradients + step) {steps_a} steps at {dt_a:.3f} s per "
                  f"slab step keeping {busy_a:.1f} threads busy; step alone on prescribed gradients {steps_b} steps at "
                  f"{dt_b:.4f} s keeping {busy_b:.1f} threads busy (BLAS pool {blas} threads, used by W @ Y only)",
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (n simulated nodes on one MI355X); "
              "--gpus must be 1.", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2105_09080_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.probe:
        print(json.dumps(run_probe()))
        return
    if args.cfg5_sweep > 0:
        run_cfg5_sweep(args.cfg5_sweep)
        return
    opts = {}
    for o in args.opt:
        name, v = o.split("=")
        opts[name] = int(v)

    topo = args.topology or inputs.CONFIGS[args.config]["topologies"][0]
    main_res = run_workload(args.config, topo, args.steps, args.warmup, opts, args.copy_probe, args.trace)
    others = []
    for item in [s for s in args.also.split(",") if s]:
        name, tp = item.split(":")
        if (name, tp) == (args.config, topo):
            continue
        steps = min(args.steps, inputs.CONFIGS[name]["T"])
        others.append(run_workload(name, tp, steps, args.warmup, opts, trace=args.trace))

    def roofline_block(r):
        key = f"{r['cfg']}/{r['topology']}"
        traffic, source = MEASURED_TRAFFIC_BYTES.get(key, (None, None))
        dom_gossip = r["dominant"] == "gossip"
        return {
            "bound": "hbm",
            "workload": r["workload"],
            "kernel": f"fused gossip step ({'; '.join(r['gossip_kernels'])})"
                      if dom_gossip else "fused global-average step (k_step_global)",
            "achieved": r["achieved_gbs"],
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": r["achieved_gbs"] / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": (f"{source}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the same command, copied from that "
                               "summary, not measured by this run") if source else None,
            "algorithmic_bytes_per_launch": r["algorithmic_bytes_per_launch"],
            "avg_launch_ms": r["gossip_ms_avg"] if dom_gossip else r["global_ms_avg"],
            "gossip_ms_by_one_peer_offset": r["gossip_ms_by_offset"],
            "global_step_avg_ms": r["global_ms_avg"],
            "global_step_gbs": r.get("global_gbs"),
            "global_step_frac": r["global_gbs"] / HBM_PEAK_GBS if r.get("global_gbs") else None,
            "iterations_timed": r["iterations"], "n_gossip": r["n_gossip"], "n_global": r["n_global"],
            "pace_controllers": r["pace_controllers"],
            "step_ms_each": [round(t, 3) for t in r["step_ms_each"]],
        }

    out = {
        "metric": "Gossip-PGA steps/s and achieved HBM GB/s (% of peak) for fused n x d step",
        "value": main_res["steps_per_s"],
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": main_res["workload"], "options": opts,
                   "iterations_timed": main_res["iterations"],
                   "step": "gpga_local_grad (counter-RNG gradients) + gpga_step (fused update + mix/average)"},
        "node_updates_per_s": main_res["steps_per_s"] * main_res["n"],
        "step_only_steps_per_s": main_res["step_only_steps_per_s"],
        "roofline": roofline_block(main_res),
        "rooflines_other_workloads": {f"{r['cfg']}/{r['topology']}": roofline_block(r) for r in others},
        "consensus_trace": main_res.get("consensus_trace"),
        "breakdown": {"grad_ms_avg": main_res["grad_ms_avg"], "step_ms_avg": main_res["step_ms_avg"],
                      "grad_write_gbs": main_res["grad_write_gbs"],
                      "n_gossip": main_res["n_gossip"], "n_global": main_res["n_global"]},
        "other_workloads": [
            {"workload": r["workload"], "steps_per_s": r["steps_per_s"], "step_only_steps_per_s": r["step_only_steps_per_s"],
             "node_updates_per_s": r["steps_per_s"] * r["n"],
             "ms_per_step": r["ms_per_step"], "gossip_ms_avg": r["gossip_ms_avg"], "global_ms_avg": r["global_ms_avg"],
             "grad_ms_avg": r["grad_ms_avg"], "achieved_gbs": r["achieved_gbs"], "frac": r["achieved_gbs"] / HBM_PEAK_GBS,
             "global_step_gbs": r.get("global_gbs"), "consensus_trace": r.get("consensus_trace")} for r in others],
    }
    if not args.no_small:
        out["small_problem"] = run_simulation_shape()
    out["paper_context"] = PAPER_CONTEXT
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, topo)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
