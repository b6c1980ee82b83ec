/*
 * gpga.h - C ABI of libgpga: the Gossip-PGA iteration for n simulated nodes on
 * one MI355X (gfx950).
 *
 * The method is Gossip SGD with Periodic Global Averaging (arXiv 2105.09080).
 * Problem statement (Sec. 1, eq. (1)): n nodes minimise (1/n) sum_i f_i(x),
 * x in R^d; node i can only evaluate stochastic gradients of its own f_i.
 * Algorithm 1 (Sec. 3), for k = 0..T-1 and every node i:
 *     g_i      = grad F_i(x_i^(k); xi_i)                  (gpga_local_grad)
 *     x_i^(k+1/2) = x_i^(k) - gamma * g_i                 \
 *     if mod(k+1, H) == 0:  x_i^(k+1) = (1/n) sum_j x_j^(k+1/2)     } gpga_step
 *     else:                 x_i^(k+1) = sum_{j in N_i} w_ij x_j^(k+1/2) /
 * with W doubly stochastic, all x_i^(0) equal.  In matrix form (App. A):
 * X <- W (X - gamma G) or X <- (1/n) 1 1^T (X - gamma G), X in R^{n x d}.
 *
 * Data layout: every state array is node-major fp32, row i = node i, with a
 * common leading dimension ld >= d (in floats).  All pointers named *_dev are
 * DEVICE pointers owned by the caller (the library never allocates or frees
 * n x d memory; it owns only the context and small scratch for reductions and
 * per-sample coefficients).  Work is enqueued on the stream given to
 * gpga_bind and is asynchronous unless stated otherwise.
 *
 * Errors: every call returns a gpga_status; nothing aborts or throws across
 * the ABI.  gpga_last_error(ctx) returns a static-lifetime-of-ctx string that
 * describes the most recent failure on that context.  Invalid arguments are
 * rejected before anything is launched.  A context is not thread-safe.
 */
#ifndef GPGA_H
#define GPGA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gpga_ctx gpga_ctx; /* opaque */

typedef enum {
    GPGA_OK = 0,
    GPGA_EINVAL = 1,  /* bad argument (size, range, alignment, NULL)           */
    GPGA_ENOMEM = 2,  /* host or device scratch allocation failed              */
    GPGA_EDEVICE = 3, /* a HIP call or kernel launch reported an error         */
    GPGA_ESTATE = 4   /* call order: buffers not bound / no problem attached   */
} gpga_status;

/* Mixing graphs.  Sec. 3: W = I turns the method into Local SGD, W = (1/n)11^T
 * into parallel SGD; H -> infinity (H = 0 here) into plain Gossip SGD. */
typedef enum {
    GPGA_TOPO_RING = 0,  /* self + two ring neighbours, weights 1/3 (|N_i| = 3, Sec. 3.3;
                            reproduces the beta values printed in Sec. 5.1)              */
    GPGA_TOPO_EXPO1 = 1, /* time-varying one-peer exponential graph (App. F.1): at
                            iteration k row i averages with row (i + 2^(k mod tau)) mod n,
                            tau = ceil(log2 n), weights 1/2                             */
    GPGA_TOPO_NONE = 2,  /* W = I                                                        */
    GPGA_TOPO_FULL = 3,  /* W = (1/n) 1 1^T : every step is a global average             */
    GPGA_TOPO_GRID = 4,  /* grid, |N_i| = 5 (Sec. 3.3; 1 - beta = O(1/n)): node a*c + b of the
                            most nearly square r x c factorisation of n (r <= c) mixes itself
                            and (a +- 1, b), (a, b +- 1), indices mod r / mod c, weights 1/5;
                            coinciding neighbours (r or c below 3) add their weights          */
    GPGA_TOPO_EXPO = 5,  /* static exponential graph (App. F.2): row i mixes itself and rows
                            i + 2^j mod n, j = 0..tau-1, tau = ceil(log2 n), weights 1/(tau+1)  */
    GPGA_TOPO_CUSTOM = 6 /* any doubly stochastic W, attached with gpga_set_mixing_csr         */
} gpga_topology;

/* Algorithm 1 "Require": learning rate gamma = lr > 0 (finite), weight matrix
 * (topology), averaging period H (H >= 1; H = 0 means never average).  momentum
 * in [0,1) selects heavy-ball SGD as used in the paper's experiments (App. F.1):
 * m <- momentum*m + g, x^(k+1/2) = x - lr*m; momentum = 0 is Algorithm 1 exactly.
 * n >= 1 nodes, d >= 1 parameters.  Binds the context to the current HIP device.
 * On success *out receives a context to be released with gpga_destroy. */
gpga_status gpga_create(gpga_ctx** out, int32_t n, int64_t d, int32_t topology,
                        int64_t H, float lr, float momentum);

/* Waits for the bound stream, frees library scratch and the context. */
gpga_status gpga_destroy(gpga_ctx* ctx);

/* Attach caller-owned device buffers, each n rows x ld floats (ld >= d):
 *   x_dev     current iterates X^(k)         (read by local_grad/step)
 *   x_new_dev receives X^(k+1)               (must not alias x_dev)
 *   m_dev     momentum buffer, updated in place (may be NULL iff momentum == 0)
 *   g_dev     stochastic gradients G^(k): written by gpga_local_grad, or by the
 *             caller itself (e.g. a real backward pass) before gpga_step
 * After each gpga_step the roles of x_dev and x_new_dev swap (gpga_current_x).
 * No two of the four arrays may overlap (EINVAL).
 * Pointers must be 4-byte aligned; 16-byte aligned pointers with ld % 4 == 0
 * take the 128-bit path.  hip_stream is a hipStream_t (NULL = default stream). */
gpga_status gpga_bind(gpga_ctx* ctx, float* x_dev, float* x_new_dev, float* m_dev,
                      float* g_dev, int64_t ld, void* hip_stream);

/* Algorithm 1 "Require": all x_i^(0) identical.  Sets every row of the live X to
 * x0_dev (d floats on the device; NULL = zeros), m to zero and k to 0. */
gpga_status gpga_reset(gpga_ctx* ctx, const float* x0_dev);

/* Constant step size gamma from now on (detaches any schedule). */
gpga_status gpga_set_lr(gpga_ctx* ctx, float lr);
gpga_status gpga_set_period(gpga_ctx* ctx, int64_t H);

/* Nesterov momentum as used for the image-classification runs (App. F.1):
 * m <- momentum*m + g, x^(k+1/2) = x - lr*(g + momentum*m) with the new m.  This
 * is Nesterov's accelerated gradient written for the look-ahead point.  on = 1
 * needs momentum > 0 (EINVAL otherwise); on = 0 returns to heavy-ball. */
gpga_status gpga_set_nesterov(gpga_ctx* ctx, int32_t on);

/* Step-size schedules gamma_k of the paper's experiments.  gamma_k is evaluated
 * on the host in double precision from the iteration counter k at every
 * gpga_step / gpga_aga_step and handed to the kernel as a float.
 *   step:       gamma_k = base_lr * factor^floor(k / period)          (Sec. 5.1:
 *               0.2 halved every 1000 iterations)
 *   milestones: k < warmup_iters: warmup_start_lr + (base_lr - warmup_start_lr) * k / warmup_iters;
 *               afterwards base_lr * factor^(number of milestones <= k)  (Sec. 5.2:
 *               warm-up over 5 epochs, divided by 10 at epochs 30, 60, 90).
 *               milestones_host: count <= 16 iteration numbers in HOST memory, copied.
 *   poly:       k < warmup_iters: base_lr * k / warmup_iters; k >= total_iters: 0;
 *               else base_lr * (1 - (k - warmup_iters)/(total_iters - warmup_iters))^power
 *               (App. F.1, language modelling: polynomial decay with warm-up).
 * gpga_lr returns the gamma that the next step will use (-1 for a NULL context). */
gpga_status gpga_lr_schedule_step(gpga_ctx* ctx, float base_lr, int64_t period, float factor);
gpga_status gpga_lr_schedule_milestones(gpga_ctx* ctx, float base_lr, int64_t warmup_iters,
                                        float warmup_start_lr, const int64_t* milestones_host,
                                        int32_t count, float factor);
gpga_status gpga_lr_schedule_poly(gpga_ctx* ctx, float base_lr, int64_t warmup_iters,
                                  int64_t total_iters, float power);
float gpga_lr(const gpga_ctx* ctx);
/* Set the iteration counter k (resume): k drives the averaging schedule, the
 * one-peer offset and the address of synthetic gradients. */
gpga_status gpga_set_iter(gpga_ctx* ctx, int64_t k);
int64_t gpga_iter(const gpga_ctx* ctx);

/* ---- local objectives f_i (the "stochastic gradient" slot of Algorithm 1) ----
 * Data arrays are device pointers, borrowed until another problem is attached. */

/* Least squares: f_i(x) = 1/(2|B|) ||A_i[B] x - b_i[B]||^2.
 * A_dev: n x M x d fp32 (row-major, dense), b_dev: n x M fp32. */
gpga_status gpga_problem_lsq(gpga_ctx* ctx, const float* A_dev, const float* b_dev, int32_t M);

/* Logistic regression (Sec. 5.1): f_i(x) = (1/|B|) sum_{m in B} ln(1 + exp(-y_m h_m^T x)).
 * feat_dev: n x M x d fp32, y_dev: n x M fp32 holding +1 / -1. */
gpga_status gpga_problem_logreg(gpga_ctx* ctx, const float* feat_dev, const float* y_dev,
                                int32_t M);

/* Logistic regression whose features are never stored: h_{i,m}[c] = mu_i[c] + zeta,
 * mu_i[c] = sqrt(mu_var) * N(seed, 3, i, 0, c), zeta = N(seed, 2, i, m, c), where
 * N(seed, tag, a, b, c) is the counter-addressed standard normal defined below.
 * y_dev: n x M fp32 labels (+1 / -1). */
gpga_status gpga_problem_logreg_virtual(gpga_ctx* ctx, uint64_t seed, const float* y_dev,
                                        int32_t M, float mu_var);

/* Synthetic gradients standing in for a network's backward pass:
 * G[i][c] = sqrt(grad_var) * N(seed, 1, i, k, c), k = current iteration.
 *
 * N(seed, tag, a, b, c): Philox4x32-10 (Salmon et al., SC'11) with key
 * (seed & 0xffffffff, seed >> 32) and counter (c / 4, a, b, tag) gives words
 * r0..r3; u_j = ((r_j >> 9) + 0.5) * 2^-23; Box-Muller:
 * (sqrt(-2 ln u0) cos 2 pi u1, sqrt(-2 ln u0) sin 2 pi u1) are columns 4*(c/4)+0,1
 * and the same with (u2, u3) columns +2,+3. */
gpga_status gpga_problem_synthetic(gpga_ctx* ctx, uint64_t seed, float grad_var);

/* g_i = grad F_i(x_i^(k); xi_i) for every node i at its own current row x_i,
 * written to g_dev.  batch_idx_dev: n x B int32 sample indices in [0, M) (the
 * minibatch xi_i, drawn by the caller); NULL with B = 0 means the full local
 * dataset.  The kernels check every index: one outside [0, M) is never used as an
 * address, and the gradient row (and loss) of its node comes out as NaN.  Ignored for the synthetic problem.  ESTATE without bind/problem. */
gpga_status gpga_local_grad(gpga_ctx* ctx, const int32_t* batch_idx_dev, int32_t B);

/* Loss companion of gpga_local_grad (used by adaptive averaging, Alg. 2):
 * loss_dev[i] = F_i(x_i^(k); xi_i) for the same minibatch, n floats on the
 * device.  Not available for the synthetic problem (EINVAL). */
gpga_status gpga_local_loss(gpga_ctx* ctx, const int32_t* batch_idx_dev, int32_t B,
                            float* loss_dev);

/* One iteration of Algorithm 1 lines 2-6 as a single fused kernel: momentum and
 * local update, then the global average if mod(k+1, H) == 0 (H > 0) or
 * topology == FULL, else one gossip step with W_k.  Reads x, m, g once, writes
 * m and x_new once; then swaps x / x_new and increments k. */
gpga_status gpga_step(gpga_ctx* ctx);

/* The loop of Algorithm 1: T iterations, each gpga_local_grad followed by
 * gpga_step, enqueued from one call (no per-iteration trip through the caller;
 * nothing synchronises).  batch_table_dev: T x n x B int32 on the device, iteration
 * j of this call uses rows [j*n*B, (j+1)*n*B); NULL with B = 0 means full batches
 * (and is what the synthetic problem takes).  Stops at the first failing call and
 * returns its status; iterations before it stay enqueued.  With adaptive averaging
 * enabled (gpga_aga_enable) every iteration is a gpga_aga_step instead, the library
 * evaluating the minibatch losses itself in the iterations that end in a global
 * average (those synchronise, as gpga_aga_step does).
 * Small problems with stored features (least squares or logistic; n*d <= 8192,
 * d <= 512, B <= 32, n*B <= 4096, n*B*d <= 2^17; the simulation of Sec. 5.1 is one) take a second form
 * of the same loop unless option "small_run" is 0: whole iterations - gradients,
 * momentum and local update, gossip step or global average, consensus trace - run
 * inside single-workgroup launches of up to 256 iterations with the state in LDS.
 * The results are the same to rounding and land where T separate steps leave them:
 * the live X (gpga_current_x) in the same one of the two bound arrays, m updated,
 * g holding the gradients of the last iteration. */
gpga_status gpga_run(gpga_ctx* ctx, int64_t T, const int32_t* batch_table_dev, int32_t B);

/* Attach an arbitrary weight matrix W (Sec. 3: W >= 0, W 1 = 1, 1^T W = 1^T,
 * w_ij > 0 only for neighbours and i = j) in compressed-row form and switch the
 * context to GPGA_TOPO_CUSTOM.  All three arrays are in HOST memory and are
 * copied: row_ptr_host has n+1 entries (row_ptr[0] = 0), row i owns entries
 * row_ptr[i] .. row_ptr[i+1]-1 of col_host (node j) and val_host (w_ij, fp32).
 * EINVAL if an index is out of range, a weight is negative or not finite, or a
 * row or column sum differs from 1 by more than 1e-5.  Synchronises the stream.
 * Gossip steps with GRID, EXPO and CUSTOM run as one fused kernel (the column
 * tile of all n rows staged in LDS, 20 B per element) while the tile fits in LDS
 * (n <= 256).  Above that, a W whose neighbours all lie within a circular distance
 * band <= 32 of their node (n >= 4 band; the grid is one: band = its width) runs, on
 * large problems, as a fused sliding-window kernel that keeps 4 band + 16 rows in LDS
 * (still 20 B per element); any other W runs as a local-update pass followed by a
 * sparse product (28 B per element).  On
 * every path g_dev is only read, and the array that held X^(k) holds unspecified
 * values after the step (as after any step: it is the target of the next one). */
gpga_status gpga_set_mixing_csr(gpga_ctx* ctx, const int64_t* row_ptr_host, const int32_t* col_host,
                                const float* val_host);

/* Connectivity beta = ||W - (1/n) 1 1^T||_2 (Assumption 3) of the context's
 * current W (for the one-peer graph: the matrix of the current iteration),
 * computed on the host by Lanczos iteration in double precision (a Krylov space of at
 * most 1024 vectors and 256 MiB: exact to ~1e-7 for n up to a few thousand; for much
 * larger n with a tiny spectral gap the value is a lower bound of beta). */
gpga_status gpga_mixing_beta(gpga_ctx* ctx, double* beta_out);
/* The same for a named graph (not CUSTOM) without a context or a device. */
gpga_status gpga_topology_beta(int32_t topology, int32_t n, int64_t k, double* beta_out);
/* Validates host CSR arrays exactly as gpga_set_mixing_csr does (EINVAL if W is
 * rejected) and, if beta_out is not NULL, stores its beta.  Needs no device. */
gpga_status gpga_check_mixing_csr(int32_t n, const int64_t* row_ptr_host, const int32_t* col_host,
                                  const float* val_host, double* beta_out);

/* Adaptive averaging period, Gossip-AGA (Algorithm 2, App. G).  After
 * gpga_aga_enable the period starts at H_init and iterations are advanced with
 * gpga_aga_step instead of gpga_step: a counter C of iterations since the last
 * global average is incremented; when C reaches the current H the step is a
 * global average, F = (1/n) sum_i loss_dev[i] is formed, and either the warm-up
 * estimate F_init <- (F_init + F)/2 is refreshed (iteration k < warmup_iters;
 * F_init starts at 0) or H <- ceil(F_init / F * H_init), kept in [1, H_max].
 * loss_dev: n floats on the device, the minibatch losses F_i(x_i^(k); xi_i) of
 * this iteration (gpga_local_loss, called before the step).  Averaging steps
 * synchronise the stream (one scalar is read back).  1 <= H_init <= H_max. */
gpga_status gpga_aga_enable(gpga_ctx* ctx, int64_t H_init, int64_t warmup_iters, int64_t H_max);
gpga_status gpga_aga_step(gpga_ctx* ctx, const float* loss_dev);
/* Current averaging period H. */
int64_t gpga_period(const gpga_ctx* ctx);

/* Consensus distance ||X^(k) - 1 xbar^T||_F (Sec. 4; App. B) of the live X.
 * Synchronises the stream; *out_host is a host double. */
gpga_status gpga_consensus_error(gpga_ctx* ctx, double* out_host);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same quantity as
 * gpga_consensus_error, from the same kernels, written as one double to out_dev (a
 * DEVICE pointer, 8-byte aligned, caller-owned) on the bound stream.  The call
 * allocates and frees nothing and does not synchronise: the per-workgroup partial sums
 * live in a static device array of 1 MiB (131072 doubles) that every GPU the library runs
 * on holds until the process ends.  Limit: one partial per 1024 columns on 16-byte
 * aligned rows with ld % 4 == 0 (d <= 134 216 704), per 256 columns otherwise
 * (d <= 33 554 432); a larger d gives EINVAL with the limit in gpga_last_error.  All
 * calls on one GPU share that GPU's array: calls that overlap there (other streams or
 * threads) race; calls queued on one stream do not.  ESTATE before gpga_bind. */
gpga_status gpga_consensus_error_static(gpga_ctx* ctx, double* out_dev);

/* Consensus trace without host synchronisation.  While a trace is attached, every
 * gpga_step / gpga_aga_step that completes iteration k < capacity also enqueues
 * trace_dev[k] = ||X^(k+1) - 1 xbar^T||_F (a double on the DEVICE, caller-owned,
 * capacity entries); the caller reads the array whenever it likes after
 * synchronising the stream itself.  After a global average the entry is exactly 0.
 * When one wavefront or workgroup of the fused gossip kernel stores whole columns (ring
 * and one-peer steps on large problems, sparse-W steps in the tile and sliding-window
 * kernels) the sums are taken from the values it stores and X is not read again;
 * otherwise one 4 B/element reduction pass follows the step.  NULL detaches. */
gpga_status gpga_set_trace(gpga_ctx* ctx, double* trace_dev, int64_t capacity);

/* xbar = (1/n) sum_i x_i (App. A notation) of the live X into xbar_dev (d floats
 * on the device, caller-owned). */
gpga_status gpga_mean(gpga_ctx* ctx, float* xbar_dev);

/* Node average of one scalar per node: out_dev[0] = (1/n) sum_i v_dev[i] (n floats in, one
 * double out, both on the DEVICE; fp64 accumulation in a fixed order).  With the losses of
 * gpga_local_loss it is the F of Algorithm 2, and at a common point xbar the global
 * objective f(xbar) = (1/n) sum_i f_i(xbar) of eq. (1).  Asynchronous on the bound stream. */
gpga_status gpga_node_mean(gpga_ctx* ctx, const float* v_dev, double* out_dev);

/* Device pointer of the live X (x_dev or x_new_dev of gpga_bind). */
gpga_status gpga_current_x(const gpga_ctx* ctx, float** x_dev_out);

/* Launch-geometry overrides for measurement sweeps; values outside the
 * documented range give EINVAL.  Names: "unroll" (rows in flight per lane: 1, 2,
 * 4, 8), "waves" (wavefronts per workgroup: 1, 2, 4, 8), "row_split" (wavefronts
 * sharing one column tile along the node axis, 0 = automatic, else 1, 2, 4, 8;
 * must not exceed "waves"), "row_lanes" (global-average kernel: lanes of a
 * wavefront spread over rows: 0 = automatic, 1, 2, 4), "xcd_swizzle" (0/1),
 * "mix_two_pass" (1 = sparse-W gossip steps always take the two-pass path),
 * "mix_spmm_lanes" (two-pass path, second pass: lanes per column tile, 0 = automatic
 * (narrower as n grows, so that a tile's rows stay in one L2), 64, 128, 256),
 * "mix_band" (sliding-window kernel for banded W: -1 = automatic (large problems whose
 * column tile of all rows does not fit in LDS), 0 = never, 1 = whenever W qualifies),
 * "mix_waves" (sparse-W tile kernel: wavefronts per workgroup, 0 = automatic, 2, 4,
 * 8, 16), "mix_lane_bytes" (sparse-W tile kernel: 0 = automatic (16-byte lanes where the
 * tile of all rows fits in LDS, else 4-byte lanes), 16 or 4 = at most that width, 8 = 8-byte
 * lanes where they fit, else 4), "mix_tile_kb" (sparse-W tile kernel: largest tile in KiB of
 * LDS, 0 = automatic (all a workgroup may have: 160 on this chip), 1..160), "small_run" (gpga_run on small problems: 1 = whole
 * iterations in single-workgroup launches (default), 0 = one kernel per stage),
 * "mix_csr_lds" (sparse-W tile kernel: 1 = copy a small W
 * into LDS (default), 0 = read it from global memory), "cycle_kernel" (row-streaming kernel for one-peer
 * steps whose cycles have 2, 4, 8 or 16 rows: -1 = automatic (large problems), 0 = never, 1 = always),
 * "pace_min_cycle" (shortest row cycle whose walk is paced, 0 = automatic (4)),
 * "blocks_per_cu" (persistent launch of the fused step: -1 = automatic, 0 = one
 * workgroup per column-tile group, k = 1..32 resident workgroups per compute unit,
 * each striding over the tile groups), "pace_gbs" (rate in GB/s of paced
 * persistent launches: -1 = automatic: every kind of launch finds its own rate, each
 * launch measuring how far its wavefronts fell behind and setting the rate of the
 * next; 0 = free running; > 0 = exactly this rate; paced wavefronts issue
 * each row batch no earlier than a common start time plus the time the whole
 * launch needs for the rows before it at that rate, which keeps the chip
 * streaming a few rows at a time). */
gpga_status gpga_set_option(gpga_ctx* ctx, const char* name, int64_t value);

/* Lets the pacing controllers settle before a measurement or a latency-critical phase.
 * Large problems run the fused step as persistent launches paced at a rate that every
 * kind of launch (gossip step per one-peer offset class, global average) finds for itself,
 * each launch setting the rate of the next; a controller needs about a dozen launches.
 * gpga_tune runs `launches` (1..4096) fused steps of every kind the context's schedule
 * contains on the bound buffers.  The iteration counter is restored; the CONTENTS of x,
 * x_new and m afterwards are unspecified (call gpga_reset or set them), g is only read.
 * Does nothing when the launches of this context are not paced.  Asynchronous. */
gpga_status gpga_tune(gpga_ctx* ctx, int32_t launches);

/* Read-only facts about the context as doubles.  Names:
 *   "pace_<field>:<kind>" and "pace_<field>:<kind>/1"  state of the pacing controller of one kind
 *       of persistent launch, for steps that read the array bound as x (no suffix) or the one
 *       bound as x_new ("/1"): the two directions of the ping-pong have controllers of their own
 *       (kind: global, ring, peer_long, peer_16, peer_8, peer_4, cycles, self, tile, band; field: rate_gbs =
 *       rate of the next launch, last_rate_gbs, last_late_us = how long after its last
 *       deadline the slowest wavefront of the most recent launch ended, last_plan_us,
 *       last_elapsed_us, launches, late_launches, hold).  Synchronises the stream.
 *   "step_path"  which kernels the most recent gpga_step / gpga_aga_step / gpga_run iteration ran as
 *       (the sizes and W decide; every path has the same semantics): 0 none yet, 1 stencil walk
 *       (ring, one-peer, W = I), 2 row-streaming one-peer kernel (short cycles), 3 global average,
 *       4 sparse W with the whole column tile in LDS, 5 sparse banded W with a sliding window,
 *       6 sparse W in two passes, 7 whole iterations in one workgroup (small problems, gpga_run);
 *   "step_paced" (1 = that launch was a paced persistent launch), "step_lane_bytes" (16, 8 or 4),
 *   "trace_fused" (1 = the consensus-trace entry of that step came from the step kernel's own
 *       sums, 0 = a reduction pass followed or no trace is attached).  These four do not synchronise.
 * EINVAL for an unknown name. */
gpga_status gpga_query(gpga_ctx* ctx, const char* name, double* value_out);

/* Measurement aid, not part of the method: a plain streaming kernel over `bytes`
 * (a multiple of 16) per array of device memory on hip_stream, with the same 128-bit
 * non-temporal accesses as the fused step.  kind 0 reads src_dev (dst_dev: any
 * 4-byte device word, left unchanged); kind 1 writes dst_dev; kind 2 copies src_dev
 * to dst_dev; kind 3 does the fused step's arithmetic on flat arrays: reads src_dev,
 * src2_dev and inout_dev, writes inout_dev and dst_dev (3 reads : 2 writes, no row
 * structure).  Unused pointers may be NULL.  blocks_per_cu = 0 launches one lane
 * per 16-byte word; k > 0 launches k workgroups of 256 lanes per compute unit that
 * stride over the words.  Timed by the caller; gives the rates of the chip against
 * which the fused step's rate is to be read.  16-byte aligned pointers; EINVAL
 * otherwise.  Needs no context. */
gpga_status gpga_probe_stream(int32_t kind, const float* src_dev, float* dst_dev, const float* src2_dev,
                              float* inout_dev, int64_t bytes, int32_t blocks_per_cu, void* hip_stream);

const char* gpga_last_error(const gpga_ctx* ctx);
const char* gpga_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GPGA_H */
