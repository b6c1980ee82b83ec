// Host-only check program for the parts of libgpga that never touch the GPU: the graph
// builders, the validation of a caller's mixing matrix, the connectivity estimate beta
// (Assumption 3) and the schedule arithmetic of Algorithm 1.  It is compiled from the very
// sources the library uses, with AddressSanitizer and UndefinedBehaviorSanitizer on the host
// side, and run by the CPU test suite: the sanitizers abort the run on any bad access, the
// printed values are compared with the oracle by the test.
//
// Output: one line per fact, "key value...".
#include <cinttypes>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "gpga_internal.hpp"
#include "gpga_schedule.hpp"

namespace {

int failures = 0;
void expect(bool ok, const char* what) {
    if (!ok) {
        std::printf("FAIL %s\n", what);
        ++failures;
    }
}

void row_col_sums(int32_t n, const HostCsr& w, double* worst_row, double* worst_col) {
    std::vector<double> cols((size_t)n, 0.0);
    *worst_row = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        double r = 0.0;
        for (int32_t p = w.ptr[i]; p < w.ptr[i + 1]; ++p) {
            r += w.val[p];
            cols[(size_t)w.col[p]] += w.val[p];
        }
        *worst_row = std::fmax(*worst_row, std::fabs(r - 1.0));
    }
    *worst_col = 0.0;
    for (double c : cols) *worst_col = std::fmax(*worst_col, std::fabs(c - 1.0));
}

void named_graphs() {
    const int32_t sizes[] = {1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 20, 31, 50, 64, 97, 100, 128, 1024};
    for (int32_t n : sizes) {
        for (int topo = 0; topo < 4; ++topo) {
            HostCsr w;
            const char* name = topo == 0 ? "ring" : topo == 1 ? "grid" : topo == 2 ? "expo" : "expo1";
            if (topo == 0) build_ring_csr(n, &w);
            if (topo == 1) build_grid_csr(n, &w);
            if (topo == 2) build_static_expo_csr(n, &w);
            const int kmax = topo == 3 ? (n >= 500 ? 2 : tau_of(n) + 1) : 1;  // every offset, and the wrap of k mod tau
            for (int k = 0; k < kmax; ++k) {
                if (topo == 3) build_one_peer_csr(n, one_peer_shift(n, k), &w);
                const char* why = validate_csr(n, w, 1e-5);
                expect(why == nullptr, why ? why : "");
                double wr, wc;
                row_col_sums(n, w, &wr, &wc);
                expect(wr <= 1e-6 && wc <= 1e-6, "row / column sums of a named graph");
                std::printf("beta %s %d %d %.12f\n", name, n, k, mixing_beta(n, w));
            }
        }
    }
    // a large ring: the builders and the validation at the scale of n itself (no spectrum: O(n) per Lanczos step is fine,
    // but 2^20 nodes are enough to walk every index path)
    HostCsr big;
    build_ring_csr(1 << 20, &big);
    expect(validate_csr(1 << 20, big, 1e-5) == nullptr, "ring of 2^20 nodes");
    std::printf("beta ring %d 0 %.12f\n", 1 << 20, mixing_beta(1 << 20, big));
}

void rejected_matrices() {
    // every way a caller's arrays can be wrong must come back as a message, never as a bad access
    const int32_t n = 6;
    HostCsr good;
    build_ring_csr(n, &good);
    std::vector<int64_t> ptr(good.ptr.begin(), good.ptr.end());
    HostCsr out;
    expect(copy_csr(n, ptr.data(), good.col.data(), good.val.data(), &out) == nullptr, "good ring copies");
    expect(validate_csr(n, out, 1e-5) == nullptr, "good ring validates");
    expect(copy_csr(n, nullptr, good.col.data(), good.val.data(), &out) != nullptr, "NULL row_ptr");
    expect(copy_csr(n, ptr.data(), nullptr, good.val.data(), &out) != nullptr, "NULL col");
    {
        auto p2 = ptr;
        p2[0] = 1;
        expect(copy_csr(n, p2.data(), good.col.data(), good.val.data(), &out) != nullptr, "row_ptr[0] != 0");
        p2 = ptr;
        p2[3] = p2[2] - 1;
        expect(copy_csr(n, p2.data(), good.col.data(), good.val.data(), &out) != nullptr, "decreasing row_ptr");
        p2 = ptr;
        for (auto& v : p2) v = 0;
        expect(copy_csr(n, p2.data(), good.col.data(), good.val.data(), &out) != nullptr, "fewer than n entries");
    }
    auto broken = [&](int which) {
        HostCsr w = good;
        if (which == 0) w.col[4] = n;           // index one past the end
        if (which == 1) w.col[4] = -1;
        if (which == 2) w.val[5] = -0.25f;
        if (which == 3) w.val[5] = NAN;
        if (which == 4) w.val[5] = INFINITY;
        if (which == 5) w.val[0] += 1e-3f;      // row and column sums off
        if (which == 6) w.ptr[n] -= 1;          // shape does not match the arrays
        if (which == 7) w.ptr.pop_back();
        if (which == 8) w.col[2] = 2;           // row 0 mixes node 2 instead of node 5: rows still sum to 1, columns do not
        return validate_csr(n, w, 1e-5);
    };
    for (int which = 0; which < 9; ++which) {
        const char* why = broken(which);
        std::printf("rejected %d %s\n", which, why ? why : "ACCEPTED");
        expect(why != nullptr, "a defective W was accepted");
    }
    // random doubly stochastic matrices (convex combinations of permutations) and random damage
    std::mt19937_64 rng(12345);
    for (int trial = 0; trial < 200; ++trial) {
        const int32_t m = 1 + (int32_t)(rng() % 40);
        std::vector<std::vector<double>> dense((size_t)m, std::vector<double>((size_t)m, 0.0));
        double wsum = 0.0;
        std::vector<double> wts(4);
        for (auto& v : wts) wsum += (v = 0.05 + (double)(rng() % 1000) / 1000.0);
        for (int t = 0; t < 4; ++t) {
            std::vector<int32_t> perm((size_t)m);
            for (int32_t i = 0; i < m; ++i) perm[(size_t)i] = i;
            for (int32_t i = m - 1; i > 0; --i) std::swap(perm[(size_t)i], perm[(size_t)(rng() % (uint64_t)(i + 1))]);
            for (int32_t i = 0; i < m; ++i) dense[(size_t)i][(size_t)perm[(size_t)i]] += wts[(size_t)t] / wsum;
        }
        std::vector<int64_t> rp(1, 0);
        std::vector<int32_t> cl;
        std::vector<float> vl;
        for (int32_t i = 0; i < m; ++i) {
            for (int32_t j = 0; j < m; ++j)
                if (dense[(size_t)i][(size_t)j] > 0.0) {
                    cl.push_back(j);
                    vl.push_back((float)dense[(size_t)i][(size_t)j]);
                }
            rp.push_back((int64_t)cl.size());
        }
        HostCsr w;
        const char* why = copy_csr(m, rp.data(), cl.data(), vl.data(), &w);
        if (!why) why = validate_csr(m, w, 1e-5);
        expect(why == nullptr, "random doubly stochastic W rejected");
        const double beta = mixing_beta(m, w);
        expect(beta >= -1e-9 && beta <= 1.0 + 1e-6, "beta of a doubly stochastic W lies in [0, 1]");
        if (trial < 8) {
            std::printf("random_w %d", m);
            for (int32_t i = 0; i < m; ++i)
                for (int32_t j = 0; j < m; ++j) std::printf(" %.9g", (double)(float)dense[(size_t)i][(size_t)j]);
            std::printf(" beta %.12f\n", beta);
        }
        // damage one entry: an index out of range must be caught by the validation, whatever its value
        if (!cl.empty()) {
            HostCsr bad = w;
            bad.col[(size_t)(rng() % bad.col.size())] = (int32_t)(m + (int32_t)(rng() % 1000));
            expect(validate_csr(m, bad, 1e-5) != nullptr, "out-of-range column accepted");
        }
    }
}

void schedules() {
    for (int32_t n : {1, 2, 3, 8, 20, 32, 64, 100, 1024, 1 << 24}) {
        std::printf("tau %d %d shifts", n, tau_of(n));
        for (int64_t k = 0; k < 14; ++k) std::printf(" %d", one_peer_shift(n, k));
        std::printf("\n");
    }
    for (int64_t H : {0, 1, 4, 6, 48}) {
        std::printf("global_steps %" PRId64, H);
        for (int64_t k = 0; k < 100; ++k)
            if (is_global_iteration(GPGA_TOPO_RING, H, k)) std::printf(" %" PRId64, k);
        std::printf("\n");
    }
    expect(is_global_iteration(GPGA_TOPO_FULL, 0, 5), "W = J averages at every iteration");
    gpga_ctx c;
    c.lr = 0.3f;
    std::printf("lr none %.9g %.9g\n", (double)scheduled_lr(&c, 0), (double)scheduled_lr(&c, 123456789));
    c.sched = SCHED_STEP;  // Sec. 5.1: 0.2 halved every 1000 iterations
    c.sched_base = 0.2;
    c.sched_factor = 0.5;
    c.sched_period = 1000;
    std::printf("lr step");
    for (int64_t k : {0, 999, 1000, 1999, 2000, 5000, 40000, 2000000}) std::printf(" %.9g", (double)scheduled_lr(&c, k));
    std::printf("\n");
    c.sched = SCHED_MILESTONES;
    c.sched_base = 0.1 * 32;
    c.sched_factor = 0.1;
    c.sched_start = 0.1;
    c.sched_warmup = 500;
    c.sched_count = 3;
    c.sched_milestones[0] = 3000;
    c.sched_milestones[1] = 6000;
    c.sched_milestones[2] = 9000;
    std::printf("lr milestones");
    for (int64_t k : {0, 1, 250, 499, 500, 2999, 3000, 6000, 8999, 9000, 1000000}) std::printf(" %.9g", (double)scheduled_lr(&c, k));
    std::printf("\n");
    c.sched = SCHED_POLY;
    c.sched_base = 4e-3;
    c.sched_warmup = 100;
    c.sched_total = 1000;
    c.sched_power = 0.5;
    std::printf("lr poly");
    for (int64_t k : {0, 50, 100, 550, 999, 1000, 5000}) std::printf(" %.9g", (double)scheduled_lr(&c, k));
    std::printf("\n");
}

}  // namespace

int main() {
    named_graphs();
    rejected_matrices();
    schedules();
    std::printf("failures %d\n", failures);
    return failures ? 1 : 0;
}
