// Host-side schedule arithmetic of the iteration, in one place so that the library's entry points
// and the host-only check program (sanitizer build) run the same code:
//   * which iterations end in a global average (Algorithm 1: mod(k+1, H) == 0; H = 0 never),
//   * the offset of the one-peer exponential graph at iteration k (App. F.1),
//   * the step size gamma_k of the attached schedule (Sec. 5.1, Sec. 5.2 / App. F.1).
#pragma once

#include <cmath>

#include "gpga_internal.hpp"

inline int tau_of(int32_t n) {  // number of offsets of the one-peer exponential graph: ceil(log2 n), at least 1
    int t = 0;
    while ((1LL << t) < n) ++t;
    return t < 1 ? 1 : t;
}

// Row i averages with row (i + one_peer_shift) mod n at iteration k; 0 means no peer (n = 1).
inline int32_t one_peer_shift(int32_t n, int64_t k) { return (int32_t)((1LL << (k % tau_of(n))) % n); }

inline bool is_global_iteration(int32_t topo, int64_t H, int64_t k) {
    return topo == GPGA_TOPO_FULL || (H > 0 && (k + 1) % H == 0);
}

// gamma_k of the attached schedule for iteration k (double arithmetic, stored as float).
inline float scheduled_lr(const gpga_ctx* c, int64_t k) {
    double lr = c->lr;
    switch (c->sched) {
        case SCHED_STEP:
            lr = c->sched_base * std::pow(c->sched_factor, (double)(k / c->sched_period));
            break;
        case SCHED_MILESTONES:
            if (k < c->sched_warmup) {
                lr = c->sched_start + (c->sched_base - c->sched_start) * ((double)k / (double)c->sched_warmup);
            } else {
                int passed = 0;
                for (int j = 0; j < c->sched_count; ++j) passed += (k >= c->sched_milestones[j]);
                lr = c->sched_base * std::pow(c->sched_factor, (double)passed);
            }
            break;
        case SCHED_POLY:
            if (k < c->sched_warmup) {
                lr = c->sched_base * ((double)k / (double)c->sched_warmup);
            } else if (k >= c->sched_total) {
                lr = 0.0;
            } else {
                const double left = 1.0 - (double)(k - c->sched_warmup) / (double)(c->sched_total - c->sched_warmup);
                lr = c->sched_base * std::pow(left, c->sched_power);
            }
            break;
        default:
            break;
    }
    return (float)lr;
}
