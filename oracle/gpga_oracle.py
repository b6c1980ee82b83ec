"""CPU oracle for the Gossip-PGA iteration (TEST INFRASTRUCTURE ONLY).

A plain, slow, float64 NumPy statement of what the accelerated path must
compute.  It exists to check the HIP library; nothing in the product path may
import it, and it imports nothing from the product package.  Only tests, the
smoke check and the CPU-baseline leg of the benchmark call into this file.

What each function follows (Gossip-PGA paper, arXiv 2105.09080):

* ``gossip_pga_step``  - Algorithm 1 (local update, then either the all-node
  mean when mod(k+1,H)=0 or one gossip step sum_j w_ij x_j^{k+1/2}), in the
  matrix form of App. A, eq. (DSGD_global_average): X <- W(X - gamma G) or
  J(X - gamma G), with a dense n x n W built explicitly.
* ``mixing_matrix``    - Sec. 3 requirements on W (non-negative, doubly
  stochastic, w_ij > 0 only for neighbours or i = j, N_i contains i).
  Ring: |N_i| = 3 (Sec. 3.3 cost model) with uniform weights 1/3, the reading
  that reproduces the beta values printed in Sec. 5.1.  One-peer exponential
  graph: App. F.1 (time-varying, one peer per iteration, equal weights).
  Grid: |N_i| = 5 (Sec. 3.3) on a torus with weights 1/5 (1 - beta = O(1/n));
  static exponential graph (App. F.2 figures): self plus the ceil(log2 n)
  power-of-two offsets with equal weights; ``custom``: any dense W.
* ``consensus_error``  - ||X - Xbar||_F, the consensus distance of Sec. 4 /
  App. B.  ``node_mean`` - xbar = (1/n) sum_i x_i (App. A notation).
* ``logreg_loss/grad`` - the logistic loss of Sec. 5.1,
  f_i(x) = (1/|B|) sum_m ln(1 + exp(-y_m h_m^T x)).
* ``lsq_loss/grad``    - f_i(x) = 1/(2|B|) ||A_i x - b_i||^2 (workload choice,
  not in the paper; fills the "stochastic gradient" slot of Algorithm 1).
* momentum             - heavy-ball as used by the paper's experiments
  (App. F.1 trains with momentum SGD; the theory, Alg. 1, is momentum-free):
  m <- mu m + g, x^{k+1/2} = x - gamma m.  mu = 0 is Algorithm 1 exactly.  The
  momentum buffer is node-local and never mixed (only model parameters are
  communicated, App. F.1).
* Nesterov momentum    - the image-classification runs use "Nesterov momentum
  SGD" (App. F.1) from the deep-learning framework the paper names; its form is
  m <- mu m + g, x^{k+1/2} = x - gamma (g + mu m), which is Nesterov's
  accelerated gradient in Sutskever's look-ahead form after the change of
  variables x = theta + mu v (pinned against that recursion).
* ``lr_*`` schedules   - step-size rules of the experiments: halving every
  1000 iterations (Sec. 5.1), linear warm-up then division by 10 at given
  epochs (Sec. 5.2 / App. F.1), polynomial decay with warm-up (App. F.1).
* ``GossipAGA``        - Algorithm 2 (App. G), the adaptive averaging period:
  a counter C of iterations since the last global average; when C reaches the
  current H the step is a global average, the minibatch losses are averaged
  over nodes, and either the warm-up estimate F_init <- (F_init + F)/2 is
  refreshed (k < K_w) or H <- ceil(F_init / F * H_init).
* counter RNG          - Philox4x32-10 (Salmon et al., SC'11) + Box-Muller,
  the generator specification shared *as a specification* with the HIP path
  (each side has its own implementation).

Parity pins (tests/test_oracle_*.py): doubly-stochastic W and mean
preservation, exact consensus after a global step, H=1 == parallel SGD against
an independent loop, mean recursion, the deviation closed form of App. B with
explicit matrix powers, printed ring beta values, exact averaging of the
one-peer graph after log2(n) steps, finite differences for both gradients, the
normal-equation solution for least squares, Philox known-answer vectors from
the generator's publication, and moments of the normals.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import expit

# ----------------------------------------------------------------------------
# schedule and topology
# ----------------------------------------------------------------------------

TOPOLOGIES = ("ring", "expo1", "none", "full", "grid", "expo", "custom")


def is_global_step(k: int, H: int) -> bool:
    """Algorithm 1: iteration k (0-based) ends in the all-node mean iff
    mod(k+1, H) = 0.  H = 0 encodes H -> infinity (never)."""
    return H > 0 and (k + 1) % H == 0


def one_peer_tau(n: int) -> int:
    """Number of distinct offsets of the one-peer exponential graph: ceil(log2 n)."""
    return max(1, math.ceil(math.log2(n))) if n > 1 else 1


def one_peer_shift(n: int, k: int) -> int:
    """Offset used at iteration k: 2^(k mod tau), reduced mod n."""
    return (1 << (k % one_peer_tau(n))) % n


def grid_shape(n: int):
    """The most nearly square r x c factorisation of n (r <= c, r the largest
    divisor of n not above sqrt(n)); a prime n gives 1 x n."""
    r = int(math.isqrt(n))
    while n % r:
        r -= 1
    return r, n // r


def mixing_matrix(topology: str, n: int, k: int = 0) -> np.ndarray:
    """Dense float64 W_k with w_ij = weight of node j's iterate in node i's mix."""
    W = np.zeros((n, n), dtype=np.float64)
    if topology == "ring":
        # self and the two ring neighbours, indices mod n, weight 1/3 each
        for i in range(n):
            for j in (i - 1, i, i + 1):
                W[i, j % n] += 1.0 / 3.0
    elif topology == "expo1":
        s = one_peer_shift(n, k)
        for i in range(n):
            W[i, i] += 0.5
            W[i, (i + s) % n] += 0.5
    elif topology == "grid":
        # |N_i| = 5 (Sec. 3.3): node (a, b) of an r x c grid, numbered a*c + b, with its
        # four neighbours (a +- 1, b), (a, b +- 1); indices wrap (torus) so that every
        # node has the same neighbourhood size, weight 1/5 each.  1 - beta = O(1/n).
        r, c = grid_shape(n)
        for a in range(r):
            for b in range(c):
                i = a * c + b
                for aa, bb in ((a, b), (a - 1, b), (a + 1, b), (a, b - 1), (a, b + 1)):
                    W[i, (aa % r) * c + (bb % c)] += 1.0 / 5.0
    elif topology == "expo":
        # static exponential graph: node i hears from i + 2^0, i + 2^1, ..., i + 2^(tau-1)
        # (mod n) and itself, tau = ceil(log2 n), equal weights 1/(tau + 1)
        tau = one_peer_tau(n)
        for i in range(n):
            W[i, i] += 1.0 / (tau + 1)
            for j in range(tau):
                W[i, (i + (1 << j)) % n] += 1.0 / (tau + 1)
    elif topology == "none":      # W = I : Local SGD
        W[np.arange(n), np.arange(n)] = 1.0
    elif topology == "full":      # W = (1/n) 1 1^T : parallel SGD
        W[:] = 1.0 / n
    else:
        raise ValueError(f"unknown topology {topology!r}")
    return W


def beta_of(W: np.ndarray) -> float:
    """beta = ||W - (1/n) 1 1^T||_2 (Assumption 3)."""
    n = W.shape[0]
    return float(np.linalg.norm(W - np.full((n, n), 1.0 / n), 2))


# ----------------------------------------------------------------------------
# the iteration
# ----------------------------------------------------------------------------

def local_update(X, Mbuf, G, lr: float, momentum: float, nesterov: bool = False):
    """m <- mu m + g ; x^{k+1/2} = x - gamma m  (Alg. 1 line 2 when mu = 0).
    Nesterov variant (App. F.1): x^{k+1/2} = x - gamma (g + mu m) with the new m."""
    X = np.asarray(X, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    if momentum == 0.0:
        M_new = G.copy()
    else:
        M_new = momentum * np.asarray(Mbuf, dtype=np.float64) + G
    if nesterov:
        return X - lr * (G + momentum * M_new), M_new
    return X - lr * M_new, M_new


def gossip_pga_step(X, Mbuf, G, k: int, *, topology: str, H: int, lr: float,
                    momentum: float = 0.0, nesterov: bool = False, W=None):
    """One iteration of Algorithm 1 in float64.  Returns (X_next, M_next).
    ``topology='custom'`` mixes with the given dense W (any doubly stochastic matrix)."""
    Y, M_new = local_update(X, Mbuf, G, lr, momentum, nesterov)
    if is_global_step(k, H):
        xbar = Y.mean(axis=0)                       # (1/n) sum_j x_j^{k+1/2}
        X_next = np.broadcast_to(xbar, Y.shape).copy()
    else:
        Wk = np.asarray(W, dtype=np.float64) if topology == "custom" else mixing_matrix(topology, Y.shape[0], k)
        X_next = Wk @ Y
    return X_next, M_new


def node_mean(X) -> np.ndarray:
    return np.asarray(X, dtype=np.float64).mean(axis=0)


def consensus_error(X) -> float:
    """||X - 1 xbar^T||_F, two-pass, float64."""
    X = np.asarray(X, dtype=np.float64)
    D = X - X.mean(axis=0, keepdims=True)
    return float(np.sqrt(np.sum(D * D)))


# ----------------------------------------------------------------------------
# step-size schedules (gamma as a function of the iteration counter k)
# ----------------------------------------------------------------------------

def lr_step_decay(k: int, base: float, period: int, factor: float) -> float:
    """gamma_k = base * factor^floor(k / period).  Sec. 5.1 runs base = 0.2,
    factor = 1/2, period = 1000 ("decreased by half for every 1000 iterations")."""
    return base * factor ** (k // period)


def _warmup(k: int, base: float, warmup_iters: int, warmup_start: float):
    """Linear warm-up: gamma rises by a constant amount per iteration from
    ``warmup_start`` at k = 0 and reaches ``base`` at k = warmup_iters."""
    return warmup_start + (base - warmup_start) * (k / warmup_iters)


def lr_warmup_milestones(k: int, base: float, warmup_iters: int, warmup_start: float,
                         milestones, factor: float) -> float:
    """Sec. 5.2 / App. F.1: warm-up over the first iterations, then gamma is
    multiplied by ``factor`` (1/10 in the paper) at each milestone iteration
    (epochs 30, 60, 90 times the iterations per epoch)."""
    if k < warmup_iters:
        return _warmup(k, base, warmup_iters, warmup_start)
    passed = sum(1 for m in milestones if k >= m)
    return base * factor ** passed


def lr_poly(k: int, base: float, warmup_iters: int, total_iters: int, power: float) -> float:
    """App. F.1 (language modelling): warm-up from 0, then polynomial decay
    base * (1 - (k - warmup)/(total - warmup))^power, zero from total_iters on."""
    if k < warmup_iters:
        return _warmup(k, base, warmup_iters, 0.0)
    if k >= total_iters:
        return 0.0
    return base * (1.0 - (k - warmup_iters) / (total_iters - warmup_iters)) ** power


# ----------------------------------------------------------------------------
# local losses and gradients
# ----------------------------------------------------------------------------

def _rows(data_i, idx_i):
    return data_i if idx_i is None else data_i[idx_i]


def lsq_loss(A, b, X, idx=None) -> np.ndarray:
    """(n,) losses 1/(2|B|) ||A_i[B] x_i - b_i[B]||^2."""
    n = X.shape[0]
    out = np.empty(n)
    for i in range(n):
        Ai = _rows(A[i], None if idx is None else idx[i]).astype(np.float64)
        bi = _rows(b[i], None if idx is None else idx[i]).astype(np.float64)
        r = Ai @ np.asarray(X[i], dtype=np.float64) - bi
        out[i] = 0.5 * np.dot(r, r) / len(bi)
    return out


def lsq_grad(A, b, X, idx=None) -> np.ndarray:
    """(n,d) gradients (1/|B|) A_i[B]^T (A_i[B] x_i - b_i[B]); idx None = all rows."""
    n, d = X.shape
    G = np.empty((n, d))
    for i in range(n):
        Ai = _rows(A[i], None if idx is None else idx[i]).astype(np.float64)
        bi = _rows(b[i], None if idx is None else idx[i]).astype(np.float64)
        r = Ai @ np.asarray(X[i], dtype=np.float64) - bi
        G[i] = Ai.T @ r / len(bi)
    return G


def logreg_loss(feat, y, X, idx=None) -> np.ndarray:
    """(n,) losses (1/|B|) sum_m ln(1 + exp(-y_m h_m^T x_i))."""
    n = X.shape[0]
    out = np.empty(n)
    for i in range(n):
        Hi = _rows(feat[i], None if idx is None else idx[i]).astype(np.float64)
        yi = _rows(y[i], None if idx is None else idx[i]).astype(np.float64)
        z = Hi @ np.asarray(X[i], dtype=np.float64)
        out[i] = np.mean(np.logaddexp(0.0, -yi * z))
    return out


def logreg_grad(feat, y, X, idx=None) -> np.ndarray:
    """(n,d) gradients -(1/|B|) sum_m y_m sigma(-y_m h_m^T x_i) h_m."""
    n, d = X.shape
    G = np.empty((n, d))
    for i in range(n):
        Hi = _rows(feat[i], None if idx is None else idx[i]).astype(np.float64)
        yi = _rows(y[i], None if idx is None else idx[i]).astype(np.float64)
        z = Hi @ np.asarray(X[i], dtype=np.float64)
        coef = -yi * expit(-yi * z) / len(yi)
        G[i] = Hi.T @ coef
    return G


# ----------------------------------------------------------------------------
# counter-based random numbers: Philox4x32-10 + Box-Muller
# ----------------------------------------------------------------------------

_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)

TAG_GRAD = 1      # synthetic gradient   : counter (c//4, node, k, TAG_GRAD)
TAG_FEAT = 2      # virtual feature noise: counter (c//4, node, sample, TAG_FEAT)
TAG_MU = 3        # virtual node shift   : counter (c//4, node, 0, TAG_MU)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32 on arrays of 32-bit counter words.

    Each round: (hi0,lo0) = M0*c0, (hi1,lo1) = M1*c2 as 64-bit products;
    new counter = (hi1^c1^k0, lo1, hi0^c3^k1, lo0); the key is bumped by the
    Weyl constants between rounds.
    """
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK32
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK32
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK32
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK32
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def _uniform23(r):
    """32-bit word -> uniform in (0,1): ((r >> 9) + 0.5) * 2^-23.

    The top 23 bits plus the half-offset need 24 significant bits, so every
    value is exactly representable in float32 and never 0 or 1."""
    return ((np.asarray(r, dtype=np.uint64) >> np.uint64(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def counter_normals(seed: int, tag: int, node, j, c4):
    """Standard normals for column quads ``c4`` (columns 4*c4 .. 4*c4+3).

    Returns an array of shape broadcast(node, j, c4) + (4,), float64.
    Words (r0,r1) -> Box-Muller pair for columns 4c4, 4c4+1; (r2,r3) -> 4c4+2, 4c4+3:
    z_even = sqrt(-2 ln u_a) cos(2 pi u_b), z_odd = sqrt(-2 ln u_a) sin(2 pi u_b).
    """
    k0, k1 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF
    r0, r1, r2, r3 = philox4x32_10(c4, node, j, tag, k0, k1)
    u0, u1, u2, u3 = _uniform23(r0), _uniform23(r1), _uniform23(r2), _uniform23(r3)
    ra = np.sqrt(-2.0 * np.log(u0))
    rb = np.sqrt(-2.0 * np.log(u2))
    ta = 2.0 * np.pi * u1
    tb = 2.0 * np.pi * u3
    return np.stack([ra * np.cos(ta), ra * np.sin(ta), rb * np.cos(tb), rb * np.sin(tb)], axis=-1)


def _normals_at_columns(seed, tag, node, j, cols):
    """Normals for arbitrary column indices ``cols`` (1-D); node, j broadcast
    against a leading axis.  Returns shape (len(node_axis), len(cols))."""
    cols = np.asarray(cols, dtype=np.int64)
    c4 = np.unique(cols // 4)
    z = counter_normals(seed, tag, np.asarray(node)[:, None], np.asarray(j)[:, None], c4[None, :])
    z = z.reshape(z.shape[0], -1)                      # (rows, 4*len(c4)) in column order
    pos = np.searchsorted(c4, cols // 4) * 4 + (cols % 4)
    return z[:, pos]


def synthetic_grad(seed: int, k: int, n: int, cols, var: float) -> np.ndarray:
    """G[i, c] ~ N(0, var) addressed by (seed, k, i, c) for the columns ``cols``."""
    nodes = np.arange(n, dtype=np.int64)
    z = _normals_at_columns(seed, TAG_GRAD, nodes, np.full(n, k, dtype=np.int64), cols)
    return math.sqrt(var) * z


def virtual_features(seed: int, node: int, samples, cols, mu_var: float) -> np.ndarray:
    """h_{i,m}[c] = mu_i[c] + zeta_{i,m}[c] for node i, samples m, columns c.

    mu_i[c] = sqrt(mu_var) * normal(seed, TAG_MU, i, 0, c); zeta = normal(seed,
    TAG_FEAT, i, m, c).  Returns (len(samples), len(cols)) float64.
    """
    samples = np.asarray(samples, dtype=np.int64)
    mu = math.sqrt(mu_var) * _normals_at_columns(seed, TAG_MU, np.array([node]), np.array([0]), cols)
    zeta = _normals_at_columns(seed, TAG_FEAT, np.full(len(samples), node), samples, cols)
    return mu + zeta


def logreg_virtual_grad(seed: int, y, X, idx, mu_var: float, chunk: int = 1 << 16) -> np.ndarray:
    """Logistic gradient with features regenerated from the counter RNG.

    Same formula as ``logreg_grad``; the feature rows are float32-rounded
    (they stand for an fp32 feature array that is never stored).
    """
    n, d = X.shape
    G = np.zeros((n, d))
    for i in range(n):
        m = np.asarray(idx[i], dtype=np.int64)
        z = np.zeros(len(m))
        for c0 in range(0, d, chunk):
            cols = np.arange(c0, min(d, c0 + chunk))
            Hc = virtual_features(seed, i, m, cols, mu_var).astype(np.float32).astype(np.float64)
            z += Hc @ np.asarray(X[i, cols], dtype=np.float64)
        yi = np.asarray(y[i], dtype=np.float64)[m]
        coef = -yi * expit(-yi * z) / len(m)
        for c0 in range(0, d, chunk):
            cols = np.arange(c0, min(d, c0 + chunk))
            Hc = virtual_features(seed, i, m, cols, mu_var).astype(np.float32).astype(np.float64)
            G[i, cols] = Hc.T @ coef
    return G


# ----------------------------------------------------------------------------
# driver: the whole loop of Algorithm 1
# ----------------------------------------------------------------------------

def _round_f32(a):
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


class GossipPGA:
    """State (X, M, k) advanced by Algorithm 1.

    ``storage='f32'``: X, M and G are rounded to float32 (round-to-nearest-even)
    whenever they are stored, as in an fp32 parameter buffer; all arithmetic
    inside a step is float64.  ``storage='f64'``: nothing is rounded (used to
    measure how far fp32 storage alone moves a trajectory).
    All x_i^(0) are equal (Algorithm 1, "Require").
    """

    def __init__(self, n: int, d: int, *, topology: str, H: int, lr,
                 momentum: float = 0.0, nesterov: bool = False, x0=None, storage: str = "f32", W=None):
        if topology not in TOPOLOGIES:
            raise ValueError(topology)
        if (topology == "custom") != (W is not None):
            raise ValueError("a dense W goes with topology='custom' and only with it")
        self.W = None if W is None else np.asarray(W, dtype=np.float64)
        self.n, self.d = n, d
        self.topology, self.H, self.momentum = topology, H, momentum
        self.lr = lr                      # a number, or a schedule k -> gamma_k
        self.nesterov = nesterov
        self.storage = storage
        x0 = np.zeros(d) if x0 is None else np.asarray(x0, dtype=np.float64)
        self.X = np.tile(x0[None, :], (n, 1))
        self.M = np.zeros((n, d))
        self.k = 0

    def _store(self, a):
        return _round_f32(a) if self.storage == "f32" else np.asarray(a, dtype=np.float64)

    def lr_at(self, k: int) -> float:
        """gamma_k; stored as float32 like every other fp32 quantity."""
        lr = self.lr(k) if callable(self.lr) else self.lr
        return float(np.float32(lr)) if self.storage == "f32" else float(lr)

    def step(self, G):
        """Consume the gradients G (n,d) of iteration k; advance to k+1."""
        G = self._store(G)
        X_next, M_next = gossip_pga_step(self.X, self.M, G, self.k, topology=self.topology,
                                         H=self.H, lr=self.lr_at(self.k), momentum=self.momentum,
                                         nesterov=self.nesterov, W=self.W)
        self.X, self.M = self._store(X_next), self._store(M_next)
        self.k += 1
        return self.X


class GossipAGA:
    """Gossip-AGA, Algorithm 2: Gossip-PGA whose period H adapts to the loss.

    Per iteration k (0-based): C <- C+1; gradients and minibatch losses F_i at the
    current rows; local (momentum) update; if C == H: C <- 0, global average,
    F = (1/n) sum_i F_i, then F_init <- (F_init + F)/2 while k < K_w, else
    H <- ceil(F_init / F * H_init); otherwise one gossip step with W_k.
    F_init starts at 0 as printed.  Readings where the listing is silent: the
    one-peer offset is driven by the iteration counter k; H is kept in
    [1, H_max] (the analysis needs a finite H_max, Corollary 1; H >= 1 keeps
    the counter test meaningful if F_init is still 0 or F is 0).
    """

    def __init__(self, n: int, d: int, *, topology: str, H_init: int, warmup_iters: int,
                 H_max: int, lr, momentum: float = 0.0, nesterov: bool = False, x0=None,
                 storage: str = "f32"):
        self.pga = GossipPGA(n, d, topology=topology, H=0, lr=lr, momentum=momentum,
                             nesterov=nesterov, x0=x0, storage=storage)
        self.H_init, self.K_w, self.H_max = int(H_init), int(warmup_iters), int(H_max)
        self.H = int(H_init)
        self.C = 0
        self.F_init = 0.0
        self.history = []        # (k, H after the update) at every global average

    @property
    def X(self):
        return self.pga.X

    @property
    def M(self):
        return self.pga.M

    @property
    def k(self):
        return self.pga.k

    def step(self, G, losses):
        """Consume gradients G (n,d) and minibatch losses (n,) of iteration k."""
        p = self.pga
        k = p.k
        self.C += 1
        G = p._store(G)
        Y, M_next = local_update(p.X, p.M, G, p.lr_at(k), p.momentum, p.nesterov)
        if self.C == self.H:
            self.C = 0
            xbar = Y.mean(axis=0)
            X_next = np.broadcast_to(xbar, Y.shape).copy()
            F = float(np.mean(np.asarray(p._store(losses), dtype=np.float64)))
            if k < self.K_w:
                self.F_init = 0.5 * (self.F_init + F)
            else:
                ratio = self.F_init / F if F > 0.0 else float("inf")
                H_new = math.ceil(ratio * self.H_init) if math.isfinite(ratio) else self.H_max
                self.H = int(min(max(H_new, 1), self.H_max))
            self.history.append((k, self.H))
        else:
            Wk = p.W if p.topology == "custom" else mixing_matrix(p.topology, p.n, k)
            X_next = Wk @ Y
        p.X, p.M = p._store(X_next), p._store(M_next)
        p.k += 1
        return p.X
