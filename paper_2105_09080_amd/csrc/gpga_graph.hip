// Host-side mixing graphs: construction of the sparse weight matrix W for the
// named topologies, validation of a caller-supplied W against the
// requirements of Sec. 3 (non-negative, doubly stochastic), and the
// connectivity measure beta = ||W - (1/n) 1 1^T||_2 of Assumption 3.
//
// All of this is O(nnz) set-up work on n x n objects; the n x d iterates never
// come near it.
#include <algorithm>
#include <cmath>
#include <map>

#include "gpga_internal.hpp"
#include "gpga_schedule.hpp"

namespace {

// Rows given as (column -> weight) maps: neighbours that coincide (small or
// degenerate graphs, "indices mod n") add their weights.
void from_rows(const std::vector<std::map<int32_t, double>>& rows, HostCsr* out) {
    out->ptr.assign(1, 0);
    out->col.clear();
    out->val.clear();
    for (const auto& r : rows) {
        for (const auto& e : r) {
            out->col.push_back(e.first);
            out->val.push_back((float)e.second);
        }
        out->ptr.push_back((int32_t)out->col.size());
    }
}

// y = W v  /  y = W^T v  in double.
void apply_w(const HostCsr& w, int32_t n, const std::vector<double>& v, std::vector<double>& y) {
    for (int32_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int32_t p = w.ptr[i]; p < w.ptr[i + 1]; ++p) s += (double)w.val[p] * v[w.col[p]];
        y[i] = s;
    }
}
void apply_wt(const HostCsr& w, int32_t n, const std::vector<double>& v, std::vector<double>& y) {
    std::fill(y.begin(), y.end(), 0.0);
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = w.ptr[i]; p < w.ptr[i + 1]; ++p) y[w.col[p]] += (double)w.val[p] * v[i];
}
void remove_mean(std::vector<double>& v) {
    double m = 0.0;
    for (double x : v) m += x;
    m /= (double)v.size();
    for (double& x : v) x -= m;
}
double dot(const std::vector<double>& a, const std::vector<double>& b) {
    double s = 0.0;
    for (size_t i = 0; i < a.size(); ++i) s += a[i] * b[i];
    return s;
}

// Largest eigenvalue of the symmetric tridiagonal matrix (alpha, beta) by
// bisection on the Sturm count.
double tridiag_max_eig(const std::vector<double>& alpha, const std::vector<double>& beta) {
    const int k = (int)alpha.size();
    double lo = alpha[0], hi = alpha[0];
    for (int i = 0; i < k; ++i) {
        const double r = (i > 0 ? std::fabs(beta[i - 1]) : 0.0) + (i + 1 < k ? std::fabs(beta[i]) : 0.0);
        lo = std::min(lo, alpha[i] - r);
        hi = std::max(hi, alpha[i] + r);
    }
    // count of eigenvalues >= x
    auto count_ge = [&](double x) {
        int cnt = 0;
        double q = alpha[0] - x;
        if (q >= 0.0) ++cnt;
        for (int i = 1; i < k; ++i) {
            const double den = (q == 0.0) ? 1e-300 : q;
            q = alpha[i] - x - beta[i - 1] * beta[i - 1] / den;
            if (q >= 0.0) ++cnt;
        }
        return cnt;
    };
    for (int it = 0; it < 200 && hi - lo > 1e-16 * std::max(1.0, std::fabs(hi)); ++it) {
        const double mid = 0.5 * (lo + hi);
        if (count_ge(mid) >= 1) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

}  // namespace

void build_ring_csr(int32_t n, HostCsr* out) {
    std::vector<std::map<int32_t, double>> rows(n);
    for (int32_t i = 0; i < n; ++i)
        for (int d = -1; d <= 1; ++d) rows[i][(int32_t)(((int64_t)i + d + n) % n)] += 1.0 / 3.0;
    from_rows(rows, out);
}

void build_one_peer_csr(int32_t n, int32_t shift, HostCsr* out) {
    std::vector<std::map<int32_t, double>> rows(n);
    for (int32_t i = 0; i < n; ++i) {
        rows[i][i] += 0.5;
        rows[i][(int32_t)(((int64_t)i + shift) % n)] += 0.5;
    }
    from_rows(rows, out);
}

// Grid: |N_i| = 5 (Sec. 3.3).  Node (a, b) of the most nearly square r x c
// factorisation of n, numbered a*c + b, mixes itself and (a +- 1, b), (a, b +- 1)
// with indices taken mod r / mod c (torus) and weight 1/5 each.
void build_grid_csr(int32_t n, HostCsr* out) {
    int32_t r = (int32_t)std::sqrt((double)n);
    while ((int64_t)(r + 1) * (r + 1) <= n) ++r;
    while (r > 1 && ((int64_t)r * r > n || n % r)) --r;
    if (r < 1) r = 1;
    const int32_t c = n / r;
    std::vector<std::map<int32_t, double>> rows(n);
    for (int32_t a = 0; a < r; ++a)
        for (int32_t b = 0; b < c; ++b) {
            auto& row = rows[(size_t)a * c + b];
            row[a * c + b] += 0.2;
            row[((a + r - 1) % r) * c + b] += 0.2;
            row[((a + 1) % r) * c + b] += 0.2;
            row[a * c + (b + c - 1) % c] += 0.2;
            row[a * c + (b + 1) % c] += 0.2;
        }
    from_rows(rows, out);
}

// Static exponential graph: node i mixes itself and the nodes i + 2^j (mod n),
// j = 0 .. tau-1, tau = ceil(log2 n), with equal weights 1/(tau + 1).
void build_static_expo_csr(int32_t n, HostCsr* out) {
    const int tau = tau_of(n);
    const double w = 1.0 / (double)(tau + 1);
    std::vector<std::map<int32_t, double>> rows(n);
    for (int32_t i = 0; i < n; ++i) {
        rows[i][i] += w;
        for (int j = 0; j < tau; ++j) rows[i][(int32_t)(((int64_t)i + (1LL << j)) % n)] += w;
    }
    from_rows(rows, out);
}

const char* validate_csr(int32_t n, const HostCsr& w, double tol) {
    if ((int64_t)w.ptr.size() != (int64_t)n + 1 || w.ptr[0] != 0) return "row_ptr must have n+1 entries starting at 0";
    for (int32_t i = 0; i < n; ++i)
        if (w.ptr[i + 1] < w.ptr[i]) return "row_ptr must be non-decreasing";
    if ((size_t)w.ptr[n] != w.col.size() || w.col.size() != w.val.size()) return "row_ptr[n] must equal the number of entries";
    std::vector<double> colsum(n, 0.0);
    for (int32_t i = 0; i < n; ++i) {
        double rs = 0.0;
        for (int32_t p = w.ptr[i]; p < w.ptr[i + 1]; ++p) {
            if (w.col[p] < 0 || w.col[p] >= n) return "column index out of range";
            if (!(w.val[p] >= 0.f) || !std::isfinite(w.val[p])) return "weights must be finite and non-negative";
            rs += w.val[p];
            colsum[w.col[p]] += w.val[p];
        }
        if (std::fabs(rs - 1.0) > tol) return "a row of W does not sum to 1";
    }
    for (int32_t j = 0; j < n; ++j)
        if (std::fabs(colsum[j] - 1.0) > tol) return "a column of W does not sum to 1";
    return nullptr;
}

double mixing_beta(int32_t n, const HostCsr& w) {
    if (n <= 1) return 0.0;
    // Lanczos with full reorthogonalisation on B = W^T W acting on vectors orthogonal
    // to 1 (W doubly stochastic maps that subspace into itself and J vanishes on it),
    // so sigma_max(W - J) = sqrt(lambda_max(B restricted)).
    int64_t K = std::min<int64_t>(n - 1, 1024);
    const int64_t mem_cap = (256ll << 20) / 8 / n;  // keep the Krylov basis under 256 MiB
    if (K > mem_cap) K = std::max<int64_t>(mem_cap, 8);
    std::vector<std::vector<double>> Q;
    std::vector<double> alpha, beta, v(n), t(n), z(n);
    // deterministic start vector with components along every mode
    uint64_t s = 0x9E3779B97F4A7C15ull;
    for (int32_t i = 0; i < n; ++i) {
        s = s * 6364136223846793005ull + 1442695040888963407ull;
        v[i] = (double)(s >> 11) / 9007199254740992.0 - 0.5;
    }
    remove_mean(v);
    double nrm = std::sqrt(dot(v, v));
    if (nrm == 0.0) return 0.0;
    for (double& x : v) x /= nrm;
    double best = 0.0;
    for (int64_t j = 0; j < K; ++j) {
        Q.push_back(v);
        apply_w(w, n, v, t);
        apply_wt(w, n, t, z);
        remove_mean(z);
        const double a = dot(z, v);
        alpha.push_back(a);
        for (int pass = 0; pass < 2; ++pass)
            for (const auto& q : Q) {
                const double c = dot(z, q);
                for (int32_t i = 0; i < n; ++i) z[i] -= c * q[i];
            }
        const double b = std::sqrt(dot(z, z));
        if ((j + 1) % 32 == 0 || b < 1e-14 || j + 1 == K) {
            const double lam = tridiag_max_eig(alpha, beta);
            const bool settled = std::fabs(lam - best) <= 1e-15 * std::max(1.0, lam) && j >= 64;
            best = std::max(best, lam);
            if (b < 1e-14 || settled) break;
        }
        beta.push_back(b);
        for (int32_t i = 0; i < n; ++i) v[i] = z[i] / b;
    }
    return std::sqrt(std::max(best, 0.0));
}

const char* copy_csr(int32_t n, const int64_t* row_ptr, const int32_t* col, const float* val, HostCsr* out) {
    if (!row_ptr || row_ptr[0] != 0) return "row_ptr must start at 0";
    for (int32_t i = 0; i < n; ++i)
        if (row_ptr[i + 1] < row_ptr[i]) return "row_ptr must be non-decreasing";
    const int64_t nnz = row_ptr[n];
    if (nnz < n || nnz > 0x7fffffffLL) return "W needs between n and 2^31-1 entries";
    if (!col || !val) return "col and val must not be NULL";
    out->ptr.resize((size_t)n + 1);
    for (int32_t i = 0; i <= n; ++i) out->ptr[i] = (int32_t)row_ptr[i];
    out->col.assign(col, col + nnz);
    out->val.assign(val, val + nnz);
    return nullptr;
}
