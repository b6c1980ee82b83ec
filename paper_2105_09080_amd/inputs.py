"""Seeded synthetic input generators and the workload table.

This module produces *data only*: problem matrices, labels, minibatch index
tables and the named workload parameters.  It contains none of the method's
arithmetic (no gradients, no mixing, no averaging, no counter RNG), so that
both the HIP path and the CPU oracle can consume exactly the same arrays
without sharing any code that computes results.

All draws come from ``numpy.random.default_rng([seed, tag])`` with a distinct
``tag`` per array, so any array can be regenerated on its own.

The workloads stand in for the paper's experiments by size and distribution
only (Sec. 5.1 logistic-regression simulation; Sec. 5.2 ResNet-50 ~25.5M
parameters; Sec. 5.3 BERT); none of the paper's datasets is used.
"""
from __future__ import annotations

import math

import numpy as np

# distinct stream tags for default_rng([seed, tag])
_TAG_XSTAR = 1
_TAG_A = 2
_TAG_BNOISE = 3
_TAG_MU = 4
_TAG_FEAT = 5
_TAG_LABELNOISE = 6
_TAG_BATCH = 7
_TAG_X0 = 8
_TAG_NODE_BIAS = 9
_TAG_VLABEL = 10
_TAG_GENERIC = 11
_TAG_SIM_XSTAR = 12
_TAG_SIM_FEAT = 13
_TAG_SIM_LABEL = 14

#: Named workloads.  ``H == 0`` encodes "never average" (H -> infinity).
#: ``topologies`` lists the mixing graphs the workload is run with.
CONFIGS = {
    "cfg1": dict(problem="lsq", n=8, d=1000, M=100, B=0, topologies=("ring",), H=4,
                 lr=0.01, momentum=0.0, T=200, seed=0, noise_std=0.01),
    "cfg2": dict(problem="logreg", n=32, d=10_000, M=2000, B=32, topologies=("expo1",), H=16,
                 lr=0.05, momentum=0.9, T=500, seed=0, mu_var=0.5, label_noise_std=0.1),
    "cfg3": dict(problem="synthetic", n=64, d=25_600_000, topologies=("ring", "expo1"), H=48,
                 lr=0.1, momentum=0.9, T=100, seed=0, grad_var=1e-3),
    "cfg4": dict(problem="synthetic", n=64, d=110_000_000, topologies=("expo1",), H=6,
                 lr=1e-4, momentum=0.9, T=50, seed=0, grad_var=1e-3),
    "cfg5": dict(problem="logreg_virtual", n=1024, d=1_000_000, M=500, B=16,
                 topologies=("ring", "expo1"), H=8, H_sweep=(1, 8, 64, 0),
                 lr=0.05, momentum=0.9, T=1000, seed=0, mu_var=0.5),
}


def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(tag)])


def lsq_problem(n: int, d: int, M: int, seed: int = 0, noise_std: float = 0.01):
    """Per-node least-squares data: A (n,M,d) f32, b (n,M) f32, xstar (d,) f32.

    A_i ~ N(0,1) entrywise, x* ~ N(0,1) entrywise, b_i = A_i x* + noise_std*N(0,1).
    The product is formed in float64 and rounded once.
    """
    xstar = _rng(seed, _TAG_XSTAR).standard_normal(d)
    A = _rng(seed, _TAG_A).standard_normal((n, M, d)).astype(np.float32)
    eps = _rng(seed, _TAG_BNOISE).standard_normal((n, M))
    b = np.einsum("imd,d->im", A.astype(np.float64), xstar) + noise_std * eps
    return A, b.astype(np.float32), xstar.astype(np.float32)


def logreg_problem(n: int, d: int, M: int, seed: int = 0, mu_var: float = 0.5,
                   label_noise_std: float = 0.1):
    """Per-node heterogeneous logistic-regression data.

    feat (n,M,d) f32 with h_{i,m} = mu_i + N(0,I_d), mu_i in R^d with iid
    N(0, mu_var) entries (node shift = heterogeneity); labels (n,M) f32 in
    {+1,-1}: y = sign(h^T x* + label_noise_std*N(0,1)), sign(0)=+1, with x* drawn
    N(0,I) and scaled to unit norm (the paper's simulation normalises its
    teacher vector, Sec. 5.1).
    """
    xstar = _rng(seed, _TAG_XSTAR).standard_normal(d)
    xstar /= np.linalg.norm(xstar)
    mu = math.sqrt(mu_var) * _rng(seed, _TAG_MU).standard_normal((n, d))
    feat = np.empty((n, M, d), dtype=np.float32)
    y = np.empty((n, M), dtype=np.float32)
    g_feat = _rng(seed, _TAG_FEAT)
    g_lab = _rng(seed, _TAG_LABELNOISE)
    for i in range(n):  # node by node keeps the float64 temporary small
        h = mu[i][None, :] + g_feat.standard_normal((M, d))
        feat[i] = h.astype(np.float32)
        s = feat[i].astype(np.float64) @ xstar + label_noise_std * g_lab.standard_normal(M)
        y[i] = np.where(s >= 0.0, 1.0, -1.0)
    return feat, y, xstar.astype(np.float32)


def logreg_simulation_problem(n: int, d: int, M: int, seed: int = 0, iid: bool = False):
    """Data of the paper's logistic-regression simulation (Sec. 5.1), as a recipe:

    every feature vector h_{i,m} ~ N(0, 10 I_d) (covariance 10 I, i.e. std sqrt(10));
    an auxiliary x*_i with N(0,1) entries, normalised to unit length, the same for
    all nodes (iid) or one per node (non-iid); u ~ U(0,1) and the label is +1 if
    u <= 1/(1 + exp(-h^T x*_i)), else -1.  The paper runs d = 10, M = 8000,
    n = 20/50/100.  Returns feat (n,M,d) f32, y (n,M) f32, xstar (n,d) f32.
    """
    gx = _rng(seed, _TAG_SIM_XSTAR)
    xs = gx.standard_normal((1 if iid else n, d))
    xs /= np.linalg.norm(xs, axis=1, keepdims=True)
    xstar = np.repeat(xs, n, axis=0) if iid else xs
    feat = (math.sqrt(10.0) * _rng(seed, _TAG_SIM_FEAT).standard_normal((n, M, d))).astype(np.float32)
    u = _rng(seed, _TAG_SIM_LABEL).random((n, M))
    p = 1.0 / (1.0 + np.exp(-np.einsum("imd,id->im", feat.astype(np.float64), xstar)))
    y = np.where(u <= p, 1.0, -1.0).astype(np.float32)
    return feat, y, xstar.astype(np.float32)


def virtual_labels(n: int, M: int, seed: int = 0):
    """Labels for the virtual-feature logistic problem: (n,M) f32 in {+1,-1}.

    The features of that problem are never materialised (they are a counter-RNG
    function evaluated inside the gradient), so labels cannot be computed from
    them here.  Instead each node i gets its own class prior p_i = 1/(1+exp(-nu_i)),
    nu_i ~ N(0,1), and y_{i,m} = +1 with probability p_i: label skew across nodes
    on top of the feature shift mu_i.
    """
    nu = _rng(seed, _TAG_NODE_BIAS).standard_normal(n)
    p = 1.0 / (1.0 + np.exp(-nu))
    u = _rng(seed, _TAG_VLABEL).random((n, M))
    return np.where(u < p[:, None], 1.0, -1.0).astype(np.float32)


def batch_indices(T: int, n: int, B: int, M: int, seed: int = 0) -> np.ndarray:
    """Minibatch table (T,n,B) int32: iid uniform on [0,M), with replacement."""
    return _rng(seed, _TAG_BATCH).integers(0, M, size=(T, n, B), dtype=np.int32)


def initial_point(d: int, seed: int | None = None) -> np.ndarray:
    """x0 (d,) f32: zeros by default (seed None), else N(0,1)."""
    if seed is None:
        return np.zeros(d, dtype=np.float32)
    return _rng(seed, _TAG_X0).standard_normal(d).astype(np.float32)


def random_state(n: int, d: int, seed: int = 0, scale: float = 1.0):
    """Three generic (n,d) f32 arrays (X, M, G) for single-step parity cases."""
    g = _rng(seed, _TAG_GENERIC)
    X = (scale * g.standard_normal((n, d))).astype(np.float32)
    Mb = (scale * g.standard_normal((n, d))).astype(np.float32)
    G = (scale * g.standard_normal((n, d))).astype(np.float32)
    return X, Mb, G


def slab_columns(d: int, n_slabs: int, width: int, align: int = 4) -> np.ndarray:
    """Sorted unique column indices of ``n_slabs`` slabs of ``width`` columns.

    Slab starts are spread evenly over [0, d-width], always including the first
    and the last ``width`` columns, aligned down to ``align``.  Used to pick the
    columns on which a large, column-separable workload is compared.
    """
    width = min(width, d)
    if n_slabs <= 1 or d <= width:
        starts = np.array([0], dtype=np.int64)
    else:
        starts = np.linspace(0, d - width, n_slabs).astype(np.int64)
        starts = (starts // align) * align
        starts[-1] = d - width
    cols = (starts[:, None] + np.arange(width, dtype=np.int64)[None, :]).ravel()
    return np.unique(cols)
