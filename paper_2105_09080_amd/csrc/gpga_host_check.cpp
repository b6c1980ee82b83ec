// Host-only check program for the parts of libgpga that never touch the GPU: the graph
// builders, the validation of a caller's mixing matrix, the connectivity estimate beta
// (Assumption 3), the schedule arithmetic of Algorithm 1 and the controller that sets the
// rate of paced launches (run here against a model of a launch).  It is compiled from the very
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
#include "gpga_pace.hpp"
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

// The pacing controller against a model of what the kernels measure.  A launch at rate r on a
// machine whose memory system sustains E for that kernel: up to E its slowest wavefront ends
// 40-65 us after its last deadline, and one launch in ten is late for no reason (150 us);
// above E it falls behind by 75 us per percent of excess.  The clock runs at 100 MHz; a launch
// moves the 32.768 GB of the 64 x 25.6M fused step.
struct PaceModel {
    std::mt19937 rng;
    double edge_gbs;
    explicit PaceModel(unsigned seed, double e) : rng(seed), edge_gbs(e) {}
    double uniform() { return (double)(rng() >> 8) / 16777216.0; }
    uint32_t lateness(double rate_gbs) {
        double us = 40.0 + 25.0 * uniform();
        if (rate_gbs > edge_gbs) us += (rate_gbs / edge_gbs - 1.0) * 100.0 * 75.0 + 20.0 * uniform();
        else if (uniform() < 0.1) us = 150.0;
        return (uint32_t)(us * 100.0);
    }
};

void pace_controller_model() {
    const double clock_hz = 1e8, bytes = 32.768e9;
    const double fp = 1e9 / clock_hz * 16.0;  // rate units per GB/s
    for (unsigned seed = 1; seed <= 6; ++seed) {
        const double e0 = 6150.0 + 70.0 * seed;  // 6220 .. 6570 GB/s
        PaceModel model(seed, e0);
        PaceState st{};
        PaceArgs p{};
        p.st = &st;
        p.rate_fixed_fp = 0;
        p.rate_init_fp = (uint32_t)(kPaceInitGbs * fp);
        p.rate_min_fp = (uint32_t)(1000.0 * fp);
        p.rate_max_fp = (uint32_t)(kPaceMaxGbs * fp);
        p.late_floor = (uint32_t)(kPaceLateFloorSeconds * clock_hz);
        int settle = -1, drop_recover = -1, rise_recover = -1, over = 0, counted = 0;
        double settled_rate = 0.0, sum_rate = 0.0;
        const int kDrop = 300, kRise = 600, kEnd = 900;
        for (int launch = 0; launch < kEnd; ++launch) {
            if (launch == kDrop) model.edge_gbs = e0 * 0.94;
            if (launch == kRise) model.edge_gbs = e0 * 0.94 * 1.05;
            const uint32_t r = st.rate_fp ? st.rate_fp : p.rate_init_fp;  // what pace_begin would take
            const double gbs = r / fp;
            const uint32_t plan = (uint32_t)(bytes / (gbs * 1e9) * clock_hz);
            pace_controller(p, r, model.lateness(gbs), plan);
            if (!st.rate_fp) st.rate_fp = r;  // a launch whose lateness decided nothing leaves the rate alone
            expect(st.rate_fp >= p.rate_min_fp && st.rate_fp <= p.rate_max_fp, "rate inside its range");
            if (settle < 0 && st.hold > 0) {
                settle = launch + 1;
                settled_rate = st.rate_fp / fp;
            }
            if (launch >= 60 && launch < kDrop) {
                sum_rate += gbs;
                ++counted;
                if (gbs > 1.015 * e0) ++over;
            }
            if (launch >= kDrop && drop_recover < 0 && gbs <= 1.0075 * model.edge_gbs) drop_recover = launch - kDrop;
            if (launch >= kRise && rise_recover < 0 && gbs >= 0.985 * model.edge_gbs) rise_recover = launch - kRise;
        }
        const double mean_rate = sum_rate / counted;
        std::printf("pace_model %u edge %.0f settle %d settled_rate %.0f mean_rate %.0f over %d of %d drop_recover %d rise_recover %d\n",
                    seed, e0, settle, settled_rate, mean_rate, over, counted, drop_recover, rise_recover);
        expect(settle > 0 && settle <= 48, "the controller brackets the edge within 48 launches");
        // two late launches in a row for no reason (one pair in a hundred) can end the first search early:
        // the first hold may start a few percent low, the short first hold and the next search repair it
        expect(settled_rate >= 0.96 * e0 && settled_rate <= 1.012 * e0, "the first held rate is near the edge");
        expect(mean_rate >= 0.985 * e0 && mean_rate <= 1.012 * e0, "the mean rate while holding sits at the edge");
        expect(over * 20 <= counted, "at most one launch in twenty runs more than 1.5 % past the edge");
        expect(drop_recover >= 0 && drop_recover <= 12, "a lower edge is followed within 12 launches");
        expect(rise_recover >= 0 && rise_recover <= 80, "a higher edge is found after the hold runs out");
    }
    // an edge beyond the range: the rate stops at the upper limit
    {
        PaceModel model(99, 9500.0);
        PaceState st{};
        PaceArgs p{};
        p.st = &st;
        p.rate_init_fp = (uint32_t)(kPaceInitGbs * fp);
        p.rate_min_fp = (uint32_t)(1000.0 * fp);
        p.rate_max_fp = (uint32_t)(kPaceMaxGbs * fp);
        p.late_floor = (uint32_t)(kPaceLateFloorSeconds * clock_hz);
        for (int launch = 0; launch < 200; ++launch) {
            const uint32_t r = st.rate_fp ? st.rate_fp : p.rate_init_fp;
            pace_controller(p, r, model.lateness(r / fp), (uint32_t)(bytes / (r / fp * 1e9) * clock_hz));
            if (!st.rate_fp) st.rate_fp = r;
        }
        std::printf("pace_model_limit %.0f\n", st.rate_fp / fp);
        expect(st.rate_fp <= p.rate_max_fp && st.rate_fp >= p.rate_max_fp - p.rate_max_fp / 64, "the rate stops at the upper limit");
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
    pace_controller_model();
    std::printf("failures %d\n", failures);
    return failures ? 1 : 0;
}
