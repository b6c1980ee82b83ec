// C ABI of libgpga (see include/gpga.h): argument validation, the averaging
// schedule of Algorithm 1 (global average iff mod(k+1, H) == 0), the one-peer
// offset schedule, scratch management and kernel dispatch.  All heavy work is
// in the kernels; the host code here decides *which* fused kernel runs.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "gpga_internal.hpp"
#include "gpga_pace.hpp"
#include "gpga_schedule.hpp"

namespace {

void set_err(gpga_ctx* c, const char* fmt, ...) {
    if (!c) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
}

gpga_status fail(gpga_ctx* c, gpga_status s, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

gpga_status hip_fail(gpga_ctx* c, hipError_t e, const char* what) {
    if (e == hipErrorOutOfMemory) return fail(c, GPGA_ENOMEM, "%s: %s", what, hipGetErrorString(e));
    return fail(c, GPGA_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

// Makes the context's device current for the duration of a call.
struct DeviceGuard {
    int prev = -1;
    bool changed = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) changed = (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard() {
        if (changed) (void)hipSetDevice(prev);
    }
};

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool is_pow2_le8(int64_t v) { return v == 1 || v == 2 || v == 4 || v == 8; }

gpga_status grow_f32(gpga_ctx* c, float** p, size_t* cap, size_t need) {
    if (*cap >= need) return GPGA_OK;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    if (*p) (void)hipFree(*p);
    *p = nullptr;
    *cap = 0;
    e = hipMalloc(reinterpret_cast<void**>(p), need * sizeof(float));
    if (e != hipSuccess) return hip_fail(c, e, "hipMalloc(scratch)");
    *cap = need;
    return GPGA_OK;
}

gpga_status grow_f64(gpga_ctx* c, double** p, size_t* cap, size_t need) {
    if (*cap >= need) return GPGA_OK;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    if (*p) (void)hipFree(*p);
    *p = nullptr;
    *cap = 0;
    e = hipMalloc(reinterpret_cast<void**>(p), need * sizeof(double));
    if (e != hipSuccess) return hip_fail(c, e, "hipMalloc(scratch)");
    *cap = need;
    return GPGA_OK;
}

bool finite_nonneg(float v) { return std::isfinite(v) && v >= 0.f; }

bool is_csr_topology(int topo) {
    return topo == GPGA_TOPO_GRID || topo == GPGA_TOPO_EXPO || topo == GPGA_TOPO_CUSTOM;
}

void free_csr_device(gpga_ctx* c) {
    if (c->csr_ptr_d) (void)hipFree(c->csr_ptr_d);
    if (c->csr_col_d) (void)hipFree(c->csr_col_d);
    if (c->csr_val_d) (void)hipFree(c->csr_val_d);
    if (c->csr_off_d) (void)hipFree(c->csr_off_d);
    if (c->csr_ellval_d) (void)hipFree(c->csr_ellval_d);
    c->csr_off_d = nullptr;
    c->csr_ellval_d = nullptr;
    c->csr_ptr_d = nullptr;
    c->csr_col_d = nullptr;
    c->csr_val_d = nullptr;
    c->csr_ready = false;
}

// Copies c->csr to the device (synchronous; set-up time only).
gpga_status upload_csr(gpga_ctx* c) {
    if (c->bound) {
        const hipError_t e = hipStreamSynchronize(c->stream);  // a running step may still read the old copy
        if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    }
    free_csr_device(c);
    const size_t np = c->csr.ptr.size(), nz = c->csr.col.size();
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->csr_ptr_d), np * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->csr_col_d), (nz ? nz : 1) * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->csr_val_d), (nz ? nz : 1) * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(c->csr_ptr_d, c->csr.ptr.data(), np * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess && nz) e = hipMemcpy(c->csr_col_d, c->csr.col.data(), nz * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess && nz) e = hipMemcpy(c->csr_val_d, c->csr.val.data(), nz * sizeof(float), hipMemcpyHostToDevice);
    // For the band kernel: circular offsets j - i of the neighbours and their weights, csr_max_row entries
    // per row (padded with weight 0), so that a row's list is one address computation away.
    c->csr_band = 0;
    c->csr_max_row = 0;
    for (int32_t i = 0; i < c->n; ++i) c->csr_max_row = std::max(c->csr_max_row, c->csr.ptr[i + 1] - c->csr.ptr[i]);
    const size_t K = (size_t)(c->csr_max_row > 0 ? c->csr_max_row : 1);
    std::vector<int32_t> off;
    std::vector<float> wts;
    const bool ell_ok = K <= 64 && K * (size_t)c->n <= ((size_t)1 << 26);
    if (ell_ok) {
        off.assign(K * (size_t)c->n, 0);
        wts.assign(K * (size_t)c->n, 0.f);
    }
    for (int32_t i = 0; i < c->n; ++i) {
        for (int32_t p2 = c->csr.ptr[i]; p2 < c->csr.ptr[i + 1]; ++p2) {
            int32_t dlt = c->csr.col[p2] - i;                 // in (-n, n)
            if (2 * dlt > c->n) dlt -= c->n;                   // shortest way round
            if (2 * dlt < -c->n) dlt += c->n;
            if (ell_ok) {
                off[(size_t)i * K + (size_t)(p2 - c->csr.ptr[i])] = dlt;
                wts[(size_t)i * K + (size_t)(p2 - c->csr.ptr[i])] = c->csr.val[p2];
            }
            const int32_t ad = dlt < 0 ? -dlt : dlt;
            if (ad > c->csr_band) c->csr_band = ad;
        }
    }
    if (ell_ok) {
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->csr_off_d), off.size() * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->csr_ellval_d), wts.size() * sizeof(float));
        if (e == hipSuccess) e = hipMemcpy(c->csr_off_d, off.data(), off.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(c->csr_ellval_d, wts.data(), wts.size() * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        free_csr_device(c);
        return hip_fail(c, e, "mixing matrix upload");
    }
    c->csr_ready = true;
    return GPGA_OK;
}

// W of a named graph at iteration k as a host CSR; false for graphs without a sparse form here.
bool named_graph_csr(int32_t topo, int32_t n, int64_t k, HostCsr* out) {
    switch (topo) {
        case GPGA_TOPO_RING: build_ring_csr(n, out); return true;
        case GPGA_TOPO_EXPO1: build_one_peer_csr(n, one_peer_shift(n, k), out); return true;
        case GPGA_TOPO_NONE: build_one_peer_csr(n, 0, out); return true;  // 1/2 + 1/2 on the diagonal
        case GPGA_TOPO_GRID: build_grid_csr(n, out); return true;
        case GPGA_TOPO_EXPO: build_static_expo_csr(n, out); return true;
        default: return false;
    }
}

constexpr double kStochasticTol = 1e-5;  // |row / column sum - 1| allowed for fp32 weights

gpga_status check_batch(gpga_ctx* c, const int32_t* idx, int32_t B, int32_t* Beff) {
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (c->problem == PROB_NONE) return fail(c, GPGA_ESTATE, "no problem attached (gpga_problem_*)");
    if (c->problem == PROB_SYNTH) {
        *Beff = 0;
        return GPGA_OK;
    }
    if (idx == nullptr) {
        if (B != 0) return fail(c, GPGA_EINVAL, "batch_idx_dev is NULL but B = %d (full batch needs B = 0)", B);
        if (c->problem == PROB_LOGREG_VIRTUAL)
            return fail(c, GPGA_EINVAL, "the virtual-feature problem needs an explicit minibatch");
        *Beff = c->M;
    } else {
        if (B < 1) return fail(c, GPGA_EINVAL, "B = %d must be >= 1 with a minibatch table", B);
        if (!aligned(idx, 4)) return fail(c, GPGA_EINVAL, "batch_idx_dev is not 4-byte aligned");
        if (c->problem == PROB_LOGREG_VIRTUAL && B > 32)
            return fail(c, GPGA_EINVAL, "virtual-feature problem supports B <= 32 (got %d)", B);
        *Beff = B;
    }
    if ((int64_t)*Beff > 65535 * 1024LL) return fail(c, GPGA_EINVAL, "batch too large");
    return GPGA_OK;
}

gpga_status run_grad(gpga_ctx* c, const int32_t* idx, int32_t B, float* loss_out) {
    int32_t Beff = 0;
    gpga_status s = check_batch(c, idx, B, &Beff);
    if (s != GPGA_OK) return s;
    if (c->n > 65535) return fail(c, GPGA_EINVAL, "the gradient kernels take n <= 65535 nodes (one grid row per node)");
    DeviceGuard guard(c->device);
    hipError_t e = hipSuccess;
    if (c->problem == PROB_SYNTH) {
        if (loss_out) return fail(c, GPGA_EINVAL, "the synthetic problem has no loss");
        e = launch_synth_grad(c);
    } else {
        s = grow_f32(c, &c->coef, &c->coef_cap, (size_t)2 * c->n * Beff);
        if (s != GPGA_OK) return s;
        if (c->problem == PROB_LOGREG_VIRTUAL) {
            size_t need = (size_t)c->n * Beff * (size_t)virtual_margin_chunks(c);
            const size_t cons = consensus_partials_needed(c);
            if (need < cons) need = cons;
            s = grow_f64(c, &c->partials, &c->partials_cap, need);
            if (s != GPGA_OK) return s;
            e = launch_virtual_grad(c, idx, Beff, loss_out);
        } else {
            e = launch_rows_grad(c, idx, idx ? Beff : 0, loss_out);
        }
    }
    if (e != hipSuccess) return hip_fail(c, e, "gradient kernel launch");
    return GPGA_OK;
}

}  // namespace

extern "C" {

const char* gpga_version(void) { return "libgpga 0.2 (gfx950)"; }

gpga_status gpga_create(gpga_ctx** out, int32_t n, int64_t d, int32_t topology, int64_t H, float lr,
                        float momentum) {
    if (!out) return GPGA_EINVAL;
    *out = nullptr;
    if (n < 1 || n > (1 << 24)) return GPGA_EINVAL;
    if (d < 1 || d > (int64_t)0xffffffffLL * 4) return GPGA_EINVAL;  // column quad index is 32-bit
    if (topology < GPGA_TOPO_RING || topology > GPGA_TOPO_CUSTOM) return GPGA_EINVAL;
    if (H < 0) return GPGA_EINVAL;
    if (!std::isfinite(lr) || lr < 0.f) return GPGA_EINVAL;
    if (!(momentum >= 0.f && momentum < 1.f)) return GPGA_EINVAL;
    gpga_ctx* c = new (std::nothrow) gpga_ctx();
    if (!c) return GPGA_ENOMEM;
    c->n = n;
    c->d = d;
    c->topo = topology;
    c->H = H;
    c->lr = lr;
    c->mu = momentum;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return GPGA_EDEVICE;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
        c->num_cus = cus;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, c->device) == hipSuccess && lds > 0)
        c->max_lds_block = lds;
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device) == hipSuccess && khz > 0)
        c->clock_hz = 1e3 * (double)khz;
    const size_t need = consensus_partials_needed(c);
    if (hipMalloc(reinterpret_cast<void**>(&c->partials), need * sizeof(double)) != hipSuccess) {
        (void)gpga_destroy(c);
        return GPGA_ENOMEM;
    }
    c->partials_cap = need;
    if (hipMalloc(reinterpret_cast<void**>(&c->pace_states), kPaceKeys * sizeof(PaceState)) == hipSuccess) {
        (void)hipMemset(c->pace_states, 0, kPaceKeys * sizeof(PaceState));
        (void)hipDeviceSynchronize();
    } else {
        c->pace_states = nullptr;  // launches simply run unpaced
    }
    {   // set-up of gpga_consensus_error_static on this device, so that its calls find the address ready
        double* static_ptr = nullptr;
        (void)static_scratch_for_device(c->device, &static_ptr);
    }
    if (hipHostMalloc(reinterpret_cast<void**>(&c->host_scalar), sizeof(double), hipHostMallocDefault) !=
        hipSuccess) {
        c->host_scalar = nullptr;
        (void)gpga_destroy(c);
        return GPGA_ENOMEM;
    }
    if (topology == GPGA_TOPO_GRID || topology == GPGA_TOPO_EXPO) {
        named_graph_csr(topology, n, 0, &c->csr);
        if (upload_csr(c) != GPGA_OK) {
            (void)gpga_destroy(c);
            return GPGA_ENOMEM;
        }
    }
    *out = c;
    return GPGA_OK;
}

gpga_status gpga_destroy(gpga_ctx* c) {
    if (!c) return GPGA_EINVAL;
    DeviceGuard guard(c->device);
    gpga_status s = GPGA_OK;
    if (c->bound && hipStreamSynchronize(c->stream) != hipSuccess) s = GPGA_EDEVICE;
    if (c->coef) (void)hipFree(c->coef);
    if (c->aga_loss) (void)hipFree(c->aga_loss);
    if (c->partials) (void)hipFree(c->partials);
    if (c->pace_states) (void)hipFree(c->pace_states);
    free_csr_device(c);
    if (c->host_scalar) (void)hipHostFree(c->host_scalar);
    delete c;
    return s;
}

gpga_status gpga_bind(gpga_ctx* c, float* x, float* x_new, float* m, float* g, int64_t ld,
                      void* hip_stream) {
    if (!c) return GPGA_EINVAL;
    if (!x || !x_new || !g) return fail(c, GPGA_EINVAL, "x, x_new and g must not be NULL");
    if (!m && c->mu != 0.f) return fail(c, GPGA_EINVAL, "m may be NULL only when momentum == 0");
    if (ld < c->d) return fail(c, GPGA_EINVAL, "ld = %lld is smaller than d = %lld", (long long)ld, (long long)c->d);
    if (!aligned(x, 4) || !aligned(x_new, 4) || !aligned(g, 4) || (m && !aligned(m, 4)))
        return fail(c, GPGA_EINVAL, "buffers must be 4-byte aligned");
    {   // the four n x ld arrays must not overlap: every kernel reads some while writing others
        const float* bufs[4] = {x, x_new, g, m};
        const char* names[4] = {"x", "x_new", "g", "m"};
        const uintptr_t span = (uintptr_t)c->n * (uintptr_t)ld * sizeof(float);
        for (int p = 0; p < 4; ++p)
            for (int q = p + 1; q < 4; ++q) {
                if (!bufs[p] || !bufs[q]) continue;
                const uintptr_t lo = reinterpret_cast<uintptr_t>(bufs[p]), hi = reinterpret_cast<uintptr_t>(bufs[q]);
                if ((lo <= hi ? hi - lo : lo - hi) < span)
                    return fail(c, GPGA_EINVAL, "%s and %s overlap", names[p], names[q]);
            }
    }
    c->x = x;
    c->x_first = x;
    c->x_new = x_new;
    c->m = m;
    c->g = g;
    c->ld = ld;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->bound = true;
    return GPGA_OK;
}

gpga_status gpga_reset(gpga_ctx* c, const float* x0_dev) {
    if (!c) return GPGA_EINVAL;
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (x0_dev && !aligned(x0_dev, 4)) return fail(c, GPGA_EINVAL, "x0 must be 4-byte aligned");
    DeviceGuard guard(c->device);
    hipError_t e = launch_fill_rows(c, c->x, x0_dev);
    if (e == hipSuccess && c->m) e = launch_fill_rows(c, c->m, nullptr);
    if (e != hipSuccess) return hip_fail(c, e, "fill kernel launch");
    c->k = 0;
    return GPGA_OK;
}

gpga_status gpga_set_lr(gpga_ctx* c, float lr) {
    if (!c) return GPGA_EINVAL;
    if (!std::isfinite(lr) || lr < 0.f) return fail(c, GPGA_EINVAL, "lr must be finite and >= 0");
    c->lr = lr;
    c->sched = SCHED_NONE;
    return GPGA_OK;
}

gpga_status gpga_set_nesterov(gpga_ctx* c, int32_t on) {
    if (!c) return GPGA_EINVAL;
    if (on != 0 && on != 1) return fail(c, GPGA_EINVAL, "on must be 0 or 1");
    if (on && c->mu == 0.f) return fail(c, GPGA_EINVAL, "Nesterov momentum needs momentum > 0");
    c->nesterov = on != 0;
    return GPGA_OK;
}

gpga_status gpga_lr_schedule_step(gpga_ctx* c, float base_lr, int64_t period, float factor) {
    if (!c) return GPGA_EINVAL;
    if (!finite_nonneg(base_lr) || !finite_nonneg(factor) || period < 1)
        return fail(c, GPGA_EINVAL, "need base_lr >= 0, factor >= 0 (finite) and period >= 1");
    c->sched = SCHED_STEP;
    c->sched_base = base_lr;
    c->sched_factor = factor;
    c->sched_period = period;
    return GPGA_OK;
}

gpga_status gpga_lr_schedule_milestones(gpga_ctx* c, float base_lr, int64_t warmup_iters, float warmup_start_lr,
                                        const int64_t* milestones_host, int32_t count, float factor) {
    if (!c) return GPGA_EINVAL;
    if (!finite_nonneg(base_lr) || !finite_nonneg(factor) || !finite_nonneg(warmup_start_lr) || warmup_iters < 0)
        return fail(c, GPGA_EINVAL, "need base_lr, warmup_start_lr, factor >= 0 (finite) and warmup_iters >= 0");
    if (count < 0 || count > kMaxMilestones || (count > 0 && !milestones_host))
        return fail(c, GPGA_EINVAL, "count must be 0..%d with a non-NULL table", kMaxMilestones);
    for (int j = 0; j < count; ++j)
        if (milestones_host[j] < 0) return fail(c, GPGA_EINVAL, "milestones must be >= 0");
    c->sched = SCHED_MILESTONES;
    c->sched_base = base_lr;
    c->sched_factor = factor;
    c->sched_start = warmup_start_lr;
    c->sched_warmup = warmup_iters;
    c->sched_count = count;
    for (int j = 0; j < count; ++j) c->sched_milestones[j] = milestones_host[j];
    return GPGA_OK;
}

gpga_status gpga_lr_schedule_poly(gpga_ctx* c, float base_lr, int64_t warmup_iters, int64_t total_iters,
                                  float power) {
    if (!c) return GPGA_EINVAL;
    if (!finite_nonneg(base_lr) || !std::isfinite(power) || power <= 0.f || warmup_iters < 0 ||
        total_iters <= warmup_iters)
        return fail(c, GPGA_EINVAL, "need base_lr >= 0, power > 0 and 0 <= warmup_iters < total_iters");
    c->sched = SCHED_POLY;
    c->sched_base = base_lr;
    c->sched_power = power;
    c->sched_warmup = warmup_iters;
    c->sched_total = total_iters;
    return GPGA_OK;
}

float gpga_lr(const gpga_ctx* c) { return c ? scheduled_lr(c, c->k) : -1.f; }

gpga_status gpga_set_period(gpga_ctx* c, int64_t H) {
    if (!c) return GPGA_EINVAL;
    if (H < 0) return fail(c, GPGA_EINVAL, "H must be >= 0 (0 = never average)");
    c->H = H;
    return GPGA_OK;
}

gpga_status gpga_set_iter(gpga_ctx* c, int64_t k) {
    if (!c) return GPGA_EINVAL;
    if (k < 0) return fail(c, GPGA_EINVAL, "k must be >= 0");
    c->k = k;
    return GPGA_OK;
}

int64_t gpga_iter(const gpga_ctx* c) { return c ? c->k : -1; }

gpga_status gpga_problem_lsq(gpga_ctx* c, const float* A, const float* b, int32_t M) {
    if (!c) return GPGA_EINVAL;
    if (!A || !b || M < 1) return fail(c, GPGA_EINVAL, "A, b must not be NULL and M >= 1");
    if (!aligned(A, 4) || !aligned(b, 4)) return fail(c, GPGA_EINVAL, "A, b must be 4-byte aligned");
    c->problem = PROB_LSQ;
    c->feat = A;
    c->tgt = b;
    c->M = M;
    return GPGA_OK;
}

gpga_status gpga_problem_logreg(gpga_ctx* c, const float* feat, const float* y, int32_t M) {
    if (!c) return GPGA_EINVAL;
    if (!feat || !y || M < 1) return fail(c, GPGA_EINVAL, "feat, y must not be NULL and M >= 1");
    if (!aligned(feat, 4) || !aligned(y, 4)) return fail(c, GPGA_EINVAL, "feat, y must be 4-byte aligned");
    c->problem = PROB_LOGREG;
    c->feat = feat;
    c->tgt = y;
    c->M = M;
    return GPGA_OK;
}

gpga_status gpga_problem_logreg_virtual(gpga_ctx* c, uint64_t seed, const float* y, int32_t M,
                                        float mu_var) {
    if (!c) return GPGA_EINVAL;
    if (!y || M < 1) return fail(c, GPGA_EINVAL, "y must not be NULL and M >= 1");
    if (!aligned(y, 4)) return fail(c, GPGA_EINVAL, "y must be 4-byte aligned");
    if (!std::isfinite(mu_var) || mu_var < 0.f) return fail(c, GPGA_EINVAL, "mu_var must be finite and >= 0");
    c->problem = PROB_LOGREG_VIRTUAL;
    c->feat = nullptr;
    c->tgt = y;
    c->M = M;
    c->seed = seed;
    c->mu_sigma = std::sqrt(mu_var);
    return GPGA_OK;
}

gpga_status gpga_problem_synthetic(gpga_ctx* c, uint64_t seed, float grad_var) {
    if (!c) return GPGA_EINVAL;
    if (!std::isfinite(grad_var) || grad_var < 0.f) return fail(c, GPGA_EINVAL, "grad_var must be finite and >= 0");
    c->problem = PROB_SYNTH;
    c->feat = nullptr;
    c->tgt = nullptr;
    c->M = 0;
    c->seed = seed;
    c->grad_sigma = std::sqrt(grad_var);
    return GPGA_OK;
}

gpga_status gpga_local_grad(gpga_ctx* c, const int32_t* batch_idx, int32_t B) {
    if (!c) return GPGA_EINVAL;
    return run_grad(c, batch_idx, B, nullptr);
}

gpga_status gpga_local_loss(gpga_ctx* c, const int32_t* batch_idx, int32_t B, float* loss_dev) {
    if (!c) return GPGA_EINVAL;
    if (!loss_dev || !aligned(loss_dev, 4)) return fail(c, GPGA_EINVAL, "loss_dev must be a 4-byte aligned device pointer");
    return run_grad(c, batch_idx, B, loss_dev);
}

// One fused iteration; `global` selects the all-node mean instead of the gossip mix.
static gpga_status run_step(gpga_ctx* c, bool global) {
    int mode = MODE_SELF;
    int32_t S = 0;
    if (!global && c->n > 1) {
        if (c->topo == GPGA_TOPO_RING) {
            mode = MODE_RING;
            S = 1;
        } else if (c->topo == GPGA_TOPO_EXPO1) {
            S = one_peer_shift(c->n, c->k);
            mode = S ? MODE_PEER : MODE_SELF;
        }
    }

    const bool csr = !global && c->n > 1 && is_csr_topology(c->topo);
    if (csr && !c->csr_ready)
        return fail(c, GPGA_ESTATE, "no mixing matrix attached (gpga_set_mixing_csr)");

    const bool vec = aligned(c->x, 16) && aligned(c->x_new, 16) && aligned(c->g, 16) &&
                     (!c->m || aligned(c->m, 16)) && (c->ld % 4 == 0);
    StepGeom ge;
    ge.x = c->x;
    ge.x_new = c->x_new;
    ge.m = c->m;
    ge.g = c->g;
    ge.ld = c->ld;
    ge.n = c->n;
    ge.lr = scheduled_lr(c, c->k);
    ge.mu = c->mu;
    const int64_t nv = vec ? c->d / 4 : 0;
    const int64_t tail = c->d - nv * 4;
    // Consensus trace of this iteration: 0 after a global average (all rows get the same
    // bits); sums produced by the fused kernel itself when it stores whole columns in
    // one vector pass; else one reduction pass over the new X.  Nothing here waits.
    const bool trace = c->trace && c->k < c->trace_cap;
    int64_t spread_count = 0;
    c->last_path = PATH_NONE;
    c->last_paced = 0;
    c->last_trace_fused = 0;
    hipError_t e = hipSuccess;
    for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {
        ge.col0 = pass == 0 ? 0 : nv * 4;
        ge.ncols = pass == 0 ? nv : tail;
        if (ge.ncols == 0) continue;
        const int v = pass == 0 ? 4 : 1;
        const bool fuse = trace && !global && tail == 0;
        e = global ? launch_step_global(c, ge, v)
                   : csr ? launch_step_csr(c, ge, v, fuse ? c->partials + 1 : nullptr, fuse ? &spread_count : nullptr)
                         : launch_step_walk(c, ge, mode, S, v, fuse ? c->partials + 1 : nullptr,
                                            fuse ? &spread_count : nullptr);
    }
    if (e != hipSuccess) return hip_fail(c, e, "step kernel launch");
    float* t = c->x;
    c->x = c->x_new;
    c->x_new = t;
    if (trace) {
        double* slot = c->trace + c->k;
        if (global) {
            e = launch_trace_store(c, c->partials, 0, slot);
        } else if (spread_count > 0) {
            c->last_trace_fused = 1;
            e = launch_trace_store(c, c->partials + 1, spread_count, slot);
        } else {
            e = launch_consensus_trace(c, slot);  // reduction pass over the live (new) X
        }
        if (e != hipSuccess) return hip_fail(c, e, "consensus trace launch");
    }
    c->k += 1;
    return GPGA_OK;
}

gpga_status gpga_set_trace(gpga_ctx* c, double* trace_dev, int64_t capacity) {
    if (!c) return GPGA_EINVAL;
    if (trace_dev && (!aligned(trace_dev, 8) || capacity < 1))
        return fail(c, GPGA_EINVAL, "trace_dev must be 8-byte aligned with capacity >= 1");
    if (trace_dev) {
        DeviceGuard guard(c->device);
        const gpga_status s = grow_f64(c, &c->partials, &c->partials_cap, consensus_partials_needed(c));
        if (s != GPGA_OK) return s;
    }
    c->trace = trace_dev;
    c->trace_cap = trace_dev ? capacity : 0;
    return GPGA_OK;
}

gpga_status gpga_step(gpga_ctx* c) {
    if (!c) return GPGA_EINVAL;
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (c->aga) return fail(c, GPGA_ESTATE, "adaptive averaging is enabled: call gpga_aga_step");
    DeviceGuard guard(c->device);
    return run_step(c, is_global_iteration(c->topo, c->H, c->k));
}

gpga_status gpga_set_mixing_csr(gpga_ctx* c, const int64_t* row_ptr_host, const int32_t* col_host,
                                const float* val_host) {
    if (!c) return GPGA_EINVAL;
    HostCsr w;
    const char* why = copy_csr(c->n, row_ptr_host, col_host, val_host, &w);
    if (!why) why = validate_csr(c->n, w, kStochasticTol);
    if (why) return fail(c, GPGA_EINVAL, "mixing matrix rejected: %s", why);
    DeviceGuard guard(c->device);
    c->csr = w;
    const gpga_status s = upload_csr(c);
    if (s != GPGA_OK) return s;
    c->topo = GPGA_TOPO_CUSTOM;
    return GPGA_OK;
}

gpga_status gpga_mixing_beta(gpga_ctx* c, double* beta_out) {
    if (!c) return GPGA_EINVAL;
    if (!beta_out) return fail(c, GPGA_EINVAL, "beta_out must not be NULL");
    if (c->topo == GPGA_TOPO_FULL) {
        *beta_out = 0.0;
        return GPGA_OK;
    }
    if (is_csr_topology(c->topo)) {
        if (!c->csr_ready) return fail(c, GPGA_ESTATE, "no mixing matrix attached (gpga_set_mixing_csr)");
        *beta_out = mixing_beta(c->n, c->csr);
        return GPGA_OK;
    }
    HostCsr w;
    named_graph_csr(c->topo, c->n, c->k, &w);
    *beta_out = mixing_beta(c->n, w);
    return GPGA_OK;
}

gpga_status gpga_topology_beta(int32_t topology, int32_t n, int64_t k, double* beta_out) {
    if (!beta_out || n < 1 || n > (1 << 24) || k < 0) return GPGA_EINVAL;
    if (topology == GPGA_TOPO_FULL) {
        *beta_out = 0.0;
        return GPGA_OK;
    }
    HostCsr w;
    if (!named_graph_csr(topology, n, k, &w)) return GPGA_EINVAL;
    *beta_out = mixing_beta(n, w);
    return GPGA_OK;
}

gpga_status gpga_check_mixing_csr(int32_t n, const int64_t* row_ptr_host, const int32_t* col_host,
                                  const float* val_host, double* beta_out) {
    if (n < 1 || n > (1 << 24)) return GPGA_EINVAL;
    HostCsr w;
    const char* why = copy_csr(n, row_ptr_host, col_host, val_host, &w);
    if (!why) why = validate_csr(n, w, kStochasticTol);
    if (why) return GPGA_EINVAL;
    if (beta_out) *beta_out = mixing_beta(n, w);
    return GPGA_OK;
}

gpga_status gpga_run(gpga_ctx* c, int64_t T, const int32_t* batch_table_dev, int32_t B) {
    if (!c) return GPGA_EINVAL;
    if (T < 0) return fail(c, GPGA_EINVAL, "T must be >= 0");
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (c->problem == PROB_NONE) return fail(c, GPGA_ESTATE, "no problem attached (gpga_problem_*)");
    DeviceGuard guard(c->device);
    const int64_t stride = batch_table_dev ? (int64_t)c->n * B : 0;
    if (c->aga) {
        // Algorithm 2: the minibatch losses are needed only in iterations that end in a global
        // average, which the counter tells beforehand
        gpga_status s = grow_f32(c, &c->aga_loss, &c->aga_loss_cap, (size_t)c->n);
        if (s != GPGA_OK) return s;
        for (int64_t j = 0; j < T; ++j) {
            const int32_t* idx = batch_table_dev ? batch_table_dev + j * stride : nullptr;
            if (c->aga_C + 1 == c->H) {
                s = run_grad(c, idx, B, c->aga_loss);
                if (s != GPGA_OK) return s;
            }
            s = run_grad(c, idx, B, nullptr);
            if (s == GPGA_OK) s = gpga_aga_step(c, c->aga_loss);
            if (s != GPGA_OK) return s;
        }
        return GPGA_OK;
    }
    if (small_run_fits(c, batch_table_dev, B)) {
        // the whole loop inside single-workgroup launches of up to kSmallRunMaxIters iterations
        int32_t Beff = 0;
        gpga_status s = check_batch(c, batch_table_dev, B, &Beff);
        if (s != GPGA_OK) return s;
        float lr[kSmallRunMaxIters];
        for (int64_t j = 0; j < T;) {
            const int32_t chunk = (int32_t)(T - j < kSmallRunMaxIters ? T - j : kSmallRunMaxIters);
            for (int32_t t = 0; t < chunk; ++t) lr[t] = scheduled_lr(c, c->k + t);
            const hipError_t e = launch_small_run(c, chunk, batch_table_dev ? batch_table_dev + j * stride : nullptr, B, lr);
            if (e != hipSuccess) return hip_fail(c, e, "small-problem kernel launch");
            c->last_path = PATH_SMALL_RUN;
            c->last_paced = 0;
            c->last_lane_bytes = 4;
            c->last_trace_fused = c->trace != nullptr;
            if (chunk % 2) {  // the launch left X where `chunk` separate steps would have: swap the roles like they do
                float* t = c->x;
                c->x = c->x_new;
                c->x_new = t;
            }
            c->k += chunk;
            j += chunk;
        }
        return GPGA_OK;
    }
    for (int64_t j = 0; j < T; ++j) {
        gpga_status s = run_grad(c, batch_table_dev ? batch_table_dev + j * stride : nullptr, B, nullptr);
        if (s != GPGA_OK) return s;
        s = run_step(c, is_global_iteration(c->topo, c->H, c->k));
        if (s != GPGA_OK) return s;
    }
    return GPGA_OK;
}

gpga_status gpga_aga_enable(gpga_ctx* c, int64_t H_init, int64_t warmup_iters, int64_t H_max) {
    if (!c) return GPGA_EINVAL;
    if (H_init < 1 || H_max < H_init || warmup_iters < 0)
        return fail(c, GPGA_EINVAL, "need 1 <= H_init <= H_max and warmup_iters >= 0");
    c->aga = true;
    c->aga_H_init = H_init;
    c->aga_warmup = warmup_iters;
    c->aga_H_max = H_max;
    c->aga_C = 0;
    c->aga_F_init = 0.0;
    c->H = H_init;
    return GPGA_OK;
}

gpga_status gpga_aga_step(gpga_ctx* c, const float* loss_dev) {
    if (!c) return GPGA_EINVAL;
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (!c->aga) return fail(c, GPGA_ESTATE, "adaptive averaging is not enabled (gpga_aga_enable)");
    if (!loss_dev || !aligned(loss_dev, 4)) return fail(c, GPGA_EINVAL, "loss_dev must be a 4-byte aligned device pointer");
    DeviceGuard guard(c->device);
    const int64_t k = c->k;
    c->aga_C += 1;
    const bool global = (c->aga_C == c->H);
    gpga_status s = run_step(c, global);
    if (s != GPGA_OK || !global) return s;
    c->aga_C = 0;
    // F = (1/n) sum_i F_i of this iteration's minibatches: one scalar back to the host
    hipError_t e = launch_mean_f32(c, loss_dev, c->n, c->partials);
    if (e == hipSuccess)
        e = hipMemcpyAsync(c->host_scalar, c->partials, sizeof(double), hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "loss average");
    const double F = *c->host_scalar;
    if (k < c->aga_warmup) {
        c->aga_F_init = 0.5 * (c->aga_F_init + F);
    } else {
        int64_t H_new = c->aga_H_max;
        if (F > 0.0) {
            const double h = std::ceil(c->aga_F_init / F * (double)c->aga_H_init);
            if (std::isfinite(h) && h < (double)c->aga_H_max) H_new = (int64_t)h;
        }
        if (H_new < 1) H_new = 1;
        c->H = H_new;
    }
    return GPGA_OK;
}

int64_t gpga_period(const gpga_ctx* c) { return c ? c->H : -1; }

gpga_status gpga_consensus_error(gpga_ctx* c, double* out_host) {
    if (!c) return GPGA_EINVAL;
    if (!out_host) return fail(c, GPGA_EINVAL, "out_host must not be NULL");
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    DeviceGuard guard(c->device);
    gpga_status s = grow_f64(c, &c->partials, &c->partials_cap, consensus_partials_needed(c));
    if (s != GPGA_OK) return s;
    size_t need = 0;
    hipError_t e = launch_consensus_sq(c, &need);
    if (e != hipSuccess) return hip_fail(c, e, "consensus kernel launch");
    e = hipMemcpyAsync(c->host_scalar, c->partials, sizeof(double), hipMemcpyDeviceToHost, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipMemcpyAsync");
    e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    *out_host = std::sqrt(*c->host_scalar);
    return GPGA_OK;
}

gpga_status gpga_mean(gpga_ctx* c, float* xbar_dev) {
    if (!c) return GPGA_EINVAL;
    if (!xbar_dev || !aligned(xbar_dev, 4)) return fail(c, GPGA_EINVAL, "xbar_dev must be a 4-byte aligned device pointer");
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    DeviceGuard guard(c->device);
    hipError_t e = launch_col_mean(c, xbar_dev);
    if (e != hipSuccess) return hip_fail(c, e, "mean kernel launch");
    return GPGA_OK;
}

gpga_status gpga_node_mean(gpga_ctx* c, const float* v_dev, double* out_dev) {
    if (!c) return GPGA_EINVAL;
    if (!v_dev || !aligned(v_dev, 4)) return fail(c, GPGA_EINVAL, "v_dev must be a 4-byte aligned device pointer");
    if (!out_dev || !aligned(out_dev, 8)) return fail(c, GPGA_EINVAL, "out_dev must be an 8-byte aligned device pointer");
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    DeviceGuard guard(c->device);
    const hipError_t e = launch_mean_f32(c, v_dev, c->n, out_dev);
    if (e != hipSuccess) return hip_fail(c, e, "node mean launch");
    return GPGA_OK;
}

gpga_status gpga_current_x(const gpga_ctx* c, float** x_dev_out) {
    if (!c || !x_dev_out) return GPGA_EINVAL;
    if (!c->bound) return GPGA_ESTATE;
    *x_dev_out = c->x;
    return GPGA_OK;
}

gpga_status gpga_set_option(gpga_ctx* c, const char* name, int64_t value) {
    if (!c || !name) return GPGA_EINVAL;
    if (!strcmp(name, "unroll")) {
        if (value != 0 && !is_pow2_le8(value)) return fail(c, GPGA_EINVAL, "unroll must be 0, 1, 2, 4 or 8");
        c->opt_unroll = (int)value;
    } else if (!strcmp(name, "waves")) {
        if (value != 0 && !is_pow2_le8(value)) return fail(c, GPGA_EINVAL, "waves must be 0, 1, 2, 4 or 8");
        if (value && c->opt_row_split > value) return fail(c, GPGA_EINVAL, "waves must be >= row_split");
        c->opt_waves = (int)value;
    } else if (!strcmp(name, "row_split")) {
        if (value != 0 && !is_pow2_le8(value)) return fail(c, GPGA_EINVAL, "row_split must be 0, 1, 2, 4 or 8");
        if (value > (c->opt_waves ? c->opt_waves : 4)) return fail(c, GPGA_EINVAL, "row_split must not exceed waves");
        c->opt_row_split = (int)value;
    } else if (!strcmp(name, "row_lanes")) {
        if (value != 0 && value != 1 && value != 2 && value != 4) return fail(c, GPGA_EINVAL, "row_lanes must be 0, 1, 2 or 4");
        c->opt_row_lanes = (int)value;
    } else if (!strcmp(name, "xcd_swizzle")) {
        if (value != 0 && value != 1) return fail(c, GPGA_EINVAL, "xcd_swizzle must be 0 or 1");
        c->opt_xcd_swizzle = (int)value;
    } else if (!strcmp(name, "mix_spmm_lanes")) {
        if (value != 0 && value != 64 && value != 128 && value != 256) return fail(c, GPGA_EINVAL, "mix_spmm_lanes must be 0, 64, 128 or 256");
        c->opt_mix_spmm_lanes = (int)value;
    } else if (!strcmp(name, "mix_tile_kb")) {
        if (value < 0 || value > 160) return fail(c, GPGA_EINVAL, "mix_tile_kb must be 0..160");
        c->opt_mix_tile_kb = (int)value;
    } else if (!strcmp(name, "mix_lane_bytes")) {
        if (value != 0 && value != 4 && value != 8 && value != 16)
            return fail(c, GPGA_EINVAL, "mix_lane_bytes must be 0, 4, 8 or 16");
        c->opt_mix_lane_bytes = (int)value;
    } else if (!strcmp(name, "mix_waves")) {
        if (value != 0 && value != 2 && value != 4 && value != 8 && value != 16)
            return fail(c, GPGA_EINVAL, "mix_waves must be 0, 2, 4, 8 or 16");
        c->opt_mix_waves = (int)value;
    } else if (!strcmp(name, "mix_two_pass")) {
        if (value != 0 && value != 1) return fail(c, GPGA_EINVAL, "mix_two_pass must be 0 or 1");
        c->opt_mix_two_pass = (int)value;
    } else if (!strcmp(name, "mix_band")) {
        if (value < -1 || value > 1) return fail(c, GPGA_EINVAL, "mix_band must be -1 (automatic), 0 or 1");
        c->opt_mix_band = (int)value;
    } else if (!strcmp(name, "small_run")) {
        if (value != 0 && value != 1) return fail(c, GPGA_EINVAL, "small_run must be 0 or 1");
        c->opt_small_run = (int)value;
    } else if (!strcmp(name, "mix_csr_lds")) {
        if (value != 0 && value != 1) return fail(c, GPGA_EINVAL, "mix_csr_lds must be 0 or 1");
        c->opt_mix_csr_lds = (int)value;
    } else if (!strcmp(name, "pace_gbs")) {
        if (value < -1 || value > 16000) return fail(c, GPGA_EINVAL, "pace_gbs must be -1 (automatic), 0 (off) or a rate up to 16000 GB/s");
        c->opt_pace_gbs = (int)value;
    } else if (!strcmp(name, "cycle_kernel")) {
        if (value < -1 || value > 1) return fail(c, GPGA_EINVAL, "cycle_kernel must be -1 (automatic), 0 or 1");
        c->opt_cycle_kernel = (int)value;
    } else if (!strcmp(name, "pace_min_cycle")) {
        if (value < 0 || value > (1 << 24)) return fail(c, GPGA_EINVAL, "pace_min_cycle must be 0 (automatic) or a row count");
        c->opt_pace_min_cycle = (int)value;
    } else if (!strcmp(name, "blocks_per_cu")) {
        if (value < -1 || value > 32) return fail(c, GPGA_EINVAL, "blocks_per_cu must be -1 (automatic), 0 (off) or 1..32");
        c->opt_blocks_per_cu = (int)value;
    } else {
        return fail(c, GPGA_EINVAL, "unknown option '%s'", name);
    }
    return GPGA_OK;
}

gpga_status gpga_probe_stream(int32_t kind, const float* src_dev, float* dst_dev, const float* src2_dev,
                              float* inout_dev, int64_t bytes, int32_t blocks_per_cu, void* hip_stream) {
    if (kind < 0 || kind > 3 || bytes < 16 || bytes % 16 || blocks_per_cu < 0) return GPGA_EINVAL;
    const bool need_src = kind != 1, need_dst = kind != 0, need_more = kind == 3;
    if (need_src && (!src_dev || !aligned(src_dev, 16))) return GPGA_EINVAL;
    if (need_dst && (!dst_dev || !aligned(dst_dev, 16))) return GPGA_EINVAL;
    if (kind == 0 && (!dst_dev || !aligned(dst_dev, 4))) return GPGA_EINVAL;  // 4-byte sink of the read probe
    if (need_more && (!src2_dev || !inout_dev || !aligned(src2_dev, 16) || !aligned(inout_dev, 16)))
        return GPGA_EINVAL;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return GPGA_EDEVICE;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int64_t count = bytes / 16;
    int64_t blocks = (count + 255) / 256;  // one 16-byte word per lane ...
    if (blocks_per_cu > 0 && blocks > (int64_t)cus * blocks_per_cu)
        blocks = (int64_t)cus * blocks_per_cu;  // ... or a capped grid that strides over the words
    if (blocks > 0x7fffffffLL) return GPGA_EINVAL;
    const hipError_t e = launch_probe_stream(kind, src_dev, dst_dev, src2_dev, inout_dev, count,
                                             kind == 0 ? dst_dev : nullptr, blocks,
                                             static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GPGA_OK : GPGA_EDEVICE;
}

gpga_status gpga_tune(gpga_ctx* c, int32_t launches) {
    if (!c) return GPGA_EINVAL;
    if (launches < 1 || launches > 4096) return fail(c, GPGA_EINVAL, "launches must be 1..4096");
    if (!c->bound) return fail(c, GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    if (c->aga) return fail(c, GPGA_ESTATE, "adaptive averaging is enabled");
    DeviceGuard guard(c->device);
    // only launches large enough to be paced have a rate to find
    if (!c->pace_states || c->opt_pace_gbs >= 0 || (int64_t)c->n * c->d * 4 < kPaceMinBytes) return GPGA_OK;
    const int64_t k_saved = c->k;
    double* const trace_saved = c->trace;
    c->trace = nullptr;
    gpga_status s = GPGA_OK;
    // every kind of step of the schedule: the gossip step (at each one-peer offset), the global average
    const int kinds = c->topo == GPGA_TOPO_EXPO1 ? tau_of(c->n) : 1;
    for (int kind = 0; kind <= kinds && s == GPGA_OK; ++kind) {
        const bool global = kind == kinds;
        if (global && c->H == 0 && c->topo != GPGA_TOPO_FULL) break;
        if (!global && c->topo == GPGA_TOPO_FULL) continue;
        for (int32_t j = 0; j < launches && s == GPGA_OK; ++j) {
            c->k = kind;  // the offset of a one-peer step follows k mod tau
            s = run_step(c, global);
        }
    }
    c->k = k_saved;
    c->trace = trace_saved;
    return s;
}

gpga_status gpga_query(gpga_ctx* c, const char* name, double* value_out) {
    if (!c) return GPGA_EINVAL;
    if (!name || !value_out) return fail(c, GPGA_EINVAL, "name and value_out must not be NULL");
    if (!strncmp(name, "pace_", 5)) {
        // "pace_<field>:<kind>[/1]": state of the pacing controller of one kind of launch, for steps that read
        // the array bound as x (no suffix) or the one bound as x_new ("/1")
        const char* colon = strchr(name, ':');
        static const char* kinds[] = {"global", "ring", "peer_long", "peer_8", "peer_4", "cycles", "self", "tile", "peer_16", "band"};
        int key = -1;
        for (int j = 0; colon && j < 10; ++j) {
            const size_t kl = strlen(kinds[j]);
            if (!strncmp(colon + 1, kinds[j], kl) && (colon[1 + kl] == 0 || !strcmp(colon + 1 + kl, "/1")))
                key = 2 * j + (colon[1 + kl] ? 1 : 0);
        }
        if (key < 0) return fail(c, GPGA_EINVAL, "unknown pacing kind in '%s'", name);
        if (!c->pace_states) return fail(c, GPGA_ESTATE, "this context has no pacing state");
        DeviceGuard guard(c->device);
        PaceState st;
        hipError_t e = c->bound ? hipStreamSynchronize(c->stream) : hipSuccess;
        if (e == hipSuccess) e = hipMemcpy(&st, c->pace_states + key, sizeof(st), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return hip_fail(c, e, "pacing state read-back");
        const double gbs_per_fp = 1.0 / pace_fp_per_gbs(c), us = 1e6 / c->clock_hz;
        const size_t len = (size_t)(colon - name);
        auto is = [&](const char* f) { return strlen(f) == len && !strncmp(name, f, len); };
        if (is("pace_rate_gbs")) *value_out = st.rate_fp * gbs_per_fp;
        else if (is("pace_last_rate_gbs")) *value_out = st.last_rate_fp * gbs_per_fp;
        else if (is("pace_launches")) *value_out = st.launches;
        else if (is("pace_late_launches")) *value_out = st.late_launches;
        else if (is("pace_last_late_us")) *value_out = st.last_late * us;
        else if (is("pace_last_plan_us")) *value_out = st.last_plan * us;
        else if (is("pace_last_elapsed_us")) *value_out = st.last_elapsed * us;
        else if (is("pace_hold")) *value_out = st.hold;
        else return fail(c, GPGA_EINVAL, "unknown pacing field in '%s'", name);
        return GPGA_OK;
    }
    if (!strcmp(name, "step_path")) *value_out = c->last_path;
    else if (!strcmp(name, "step_paced")) *value_out = c->last_paced;
    else if (!strcmp(name, "step_lane_bytes")) *value_out = c->last_lane_bytes;
    else if (!strcmp(name, "trace_fused")) *value_out = c->last_trace_fused;
    else return fail(c, GPGA_EINVAL, "unknown query '%s'", name);
    return GPGA_OK;
}

const char* gpga_last_error(const gpga_ctx* c) { return c ? c->err : "null context"; }

}  // extern "C"
