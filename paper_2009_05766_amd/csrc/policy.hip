// Communication policy generation (Algorithm 3 of the NetMax paper): host code, no GPU work.
// Grid search over the consensus weight rho in (0, 0.5/alpha] and the global mean iteration time tbar in
// (L, U] (Appendix A); for every grid point the linear program (lp0) is solved row by row, Y_P = E[D^T D]
// (Eq. (d2)) is formed, its second largest eigenvalue gives T_convergence = tbar ln(eps) / ln(lambda_2);
// the candidate with the smallest T_convergence wins.
//
// The linear program min sum_i p_ii s.t. (o2)-(o5) separates by rows.  For one row, with lb_m the lower
// bound of (o3) on neighbour m, the free probability mass C = 1 - sum lb and the time still to be placed
// Tb = M tbar - sum t_m lb_m, the smallest self probability is C - min(C, Tb / t_min).  The optimum is not
// unique; the point with the least-squares distance to the lower bounds is returned (it is unique and
// spreads the free mass evenly over equally fast links).  Its optimality conditions are
// q_m = max(0, mu + nu t_m): the support is a set of fastest or of slowest links, found with prefix sums.
#include "../../include/netmax.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <string>
#include <vector>

namespace {

struct RowScratch {
    std::vector<int> nb, order;
    std::vector<double> tn, lo, s0, s1, s2, q;
};

// One row.  Returns false if the row has no feasible point.
bool solve_row(int M, int i, const double *t_row, const uint8_t *d_row, const double *lb_row, double target,
               double *p_row, RowScratch &w)
{
    w.nb.clear();
    for (int m = 0; m < M; ++m)
        if (m != i && d_row[m]) w.nb.push_back(m);
    const int n = (int)w.nb.size();
    if (n == 0) return false;
    w.tn.resize(n); w.lo.resize(n); w.q.assign(n, 0.0);
    double lb_sum = 0.0, lb_time = 0.0, t_min = INFINITY, t_max = 0.0;
    for (int a = 0; a < n; ++a) {
        w.tn[a] = t_row[w.nb[a]];
        w.lo[a] = lb_row[w.nb[a]];
        lb_sum += w.lo[a];
        lb_time += w.tn[a] * w.lo[a];
        t_min = std::min(t_min, w.tn[a]);
        t_max = std::max(t_max, w.tn[a]);
    }
    const double tol = 1e-12;
    const double free_mass = 1.0 - lb_sum, free_time = target - lb_time;
    if (free_mass < -tol || free_time < -tol * std::max(1.0, target)) return false;
    if (free_time > free_mass * t_max * (1.0 + 1e-12) + tol) return false;
    const double placed = t_min > 0.0 ? std::min(std::max(free_mass, 0.0), std::max(free_time, 0.0) / t_min)
                                      : std::max(free_mass, 0.0);
    const double self = std::max(free_mass - placed, 0.0);
    const double c_mass = placed, c_time = std::max(free_time, 0.0);

    if (c_mass > 1e-13) {
        w.order.resize(n);
        std::iota(w.order.begin(), w.order.end(), 0);
        std::stable_sort(w.order.begin(), w.order.end(), [&](int a, int b) { return w.tn[a] < w.tn[b]; });
        w.s0.assign(n + 1, 0.0); w.s1.assign(n + 1, 0.0); w.s2.assign(n + 1, 0.0);
        for (int a = 0; a < n; ++a) {
            const double tv = w.tn[w.order[a]];
            w.s0[a + 1] = w.s0[a] + 1.0;
            w.s1[a + 1] = w.s1[a] + tv;
            w.s2[a + 1] = w.s2[a] + tv * tv;
        }
        const double scale = std::max(1.0, t_max);
        double best = INFINITY, best_mu = 0.0, best_nu = 0.0;
        int best_lo = 0, best_hi = 0;
        for (int j = 1; j <= n; ++j) {
            for (int side = 0; side < 2; ++side) {
                const int lo = side == 0 ? 0 : n - j, hi = lo + j;         // support = sorted positions [lo, hi)
                const double c0 = w.s0[hi] - w.s0[lo], c1 = w.s1[hi] - w.s1[lo], c2 = w.s2[hi] - w.s2[lo];
                const double det = c0 * c2 - c1 * c1;
                double mu, nu;
                if (det > 1e-12 * c0 * c2) {
                    mu = (c_mass * c2 - c_time * c1) / det;
                    nu = (c0 * c_time - c1 * c_mass) / det;
                } else {                                                   // all times in the support are equal
                    mu = c_mass / c0;
                    nu = 0.0;
                }
                const double t_lo = w.tn[w.order[lo]], t_hi = w.tn[w.order[hi - 1]];
                const double mass_err = std::fabs(mu * c0 + nu * c1 - c_mass);
                const double time_err = std::fabs(mu * c1 + nu * c2 - c_time) / scale;
                const double neg = std::max(0.0, -std::min(mu + nu * t_lo, mu + nu * t_hi));
                double outside = 0.0;
                if (lo > 0) outside = std::max(outside, mu + nu * w.tn[w.order[lo - 1]]);
                if (lo > 0) outside = std::max(outside, mu + nu * w.tn[w.order[0]]);
                if (hi < n) outside = std::max(outside, mu + nu * w.tn[w.order[hi]]);
                if (hi < n) outside = std::max(outside, mu + nu * w.tn[w.order[n - 1]]);
                const double violation = std::max(std::max(mass_err, time_err), std::max(neg, outside));
                if (violation < best) {
                    best = violation; best_mu = mu; best_nu = nu; best_lo = lo; best_hi = hi;
                }
            }
        }
        if (best > 1e-9 * std::max(1.0, c_mass)) return false;
        for (int a = best_lo; a < best_hi; ++a) w.q[w.order[a]] = std::max(0.0, best_mu + best_nu * w.tn[w.order[a]]);
    }
    for (int m = 0; m < M; ++m) p_row[m] = 0.0;
    for (int a = 0; a < n; ++a) p_row[w.nb[a]] = w.lo[a] + w.q[a];
    p_row[i] = self;
    return true;
}

// Eigenvalues of a symmetric matrix by cyclic Jacobi rotations (A is destroyed).  Ascending order.
void symmetric_eigenvalues(int n, std::vector<double> &A, std::vector<double> &ev)
{
    for (int sweep = 0; sweep < 100; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int p = 0; p < n; ++p) {
            diag += A[(size_t)p * n + p] * A[(size_t)p * n + p];
            for (int q = p + 1; q < n; ++q) off += A[(size_t)p * n + q] * A[(size_t)p * n + q];
        }
        if (off <= 1e-30 * std::max(diag, 1e-300)) break;
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                const double apq = A[(size_t)p * n + q];
                if (apq == 0.0) continue;
                const double app = A[(size_t)p * n + p], aqq = A[(size_t)q * n + q];
                const double theta = (aqq - app) / (2.0 * apq);
                const double tt = (theta >= 0.0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(tt * tt + 1.0), s = tt * c;
                for (int k = 0; k < n; ++k) {       // columns p, q
                    const double akp = A[(size_t)k * n + p], akq = A[(size_t)k * n + q];
                    A[(size_t)k * n + p] = c * akp - s * akq;
                    A[(size_t)k * n + q] = s * akp + c * akq;
                }
                for (int k = 0; k < n; ++k) {       // rows p, q
                    const double apk = A[(size_t)p * n + k], aqk = A[(size_t)q * n + k];
                    A[(size_t)p * n + k] = c * apk - s * aqk;
                    A[(size_t)q * n + k] = s * apk + c * aqk;
                }
            }
    }
    ev.resize(n);
    for (int p = 0; p < n; ++p) ev[p] = A[(size_t)p * n + p];
    std::sort(ev.begin(), ev.end());
}

}  // namespace

extern "C" int netmax_generate_policy(int32_t M, const double *t_host, const uint8_t *adj, double alpha, int32_t K,
                                      int32_t R, double eps, double *P_out, double *rho_out, double *tbar_out,
                                      double *lambda2_out, double *t_conv_out)
{
    if (M < 2 || M > 4096 || !t_host || !P_out || !rho_out || !(alpha > 0.0) || K < 1 || R < 1 || !(eps > 0.0) || !(eps < 1.0))
        return NETMAX_EINVAL;
    const size_t mm = (size_t)M * M;
    std::vector<uint8_t> d(mm, 1);
    for (int i = 0; i < M; ++i)
        for (int m = 0; m < M; ++m) d[(size_t)i * M + m] = (i != m) && (!adj || adj[(size_t)i * M + m]);
    for (size_t e = 0; e < mm; ++e)
        if (!(t_host[e] >= 0.0) || !std::isfinite(t_host[e])) return NETMAX_EINVAL;

    std::vector<double> lb(mm), P(mm), Y(mm), best_P, ev, act(M), a1(mm), a2(mm);
    RowScratch scratch;
    bool found = false;
    double best_conv = INFINITY;
    const double u_rho = 0.5 / alpha;
    for (int k = 1; k <= K; ++k) {
        const double rho = u_rho * (double)k / (double)K;
        // interval of tbar: Eq. (oa3), (oa5)
        double L = 0.0, U = INFINITY;
        for (int i = 0; i < M; ++i) {
            double li = 0.0, ui = 0.0;
            for (int m = 0; m < M; ++m) {
                const size_t e = (size_t)i * M + m;
                const int both = d[e] + d[(size_t)m * M + i];
                lb[e] = d[e] ? alpha * rho * both : 0.0;
                if (d[e]) {
                    li += t_host[e] * both;
                    ui = std::max(ui, t_host[e]);
                }
            }
            L = std::max(L, alpha * rho / M * li);
            U = std::min(U, ui / M);
        }
        if (!(L <= U)) continue;
        for (int r = 1; r <= R; ++r) {
            const double tbar = L + (U - L) * (double)r / (double)R;
            bool ok = true;
            for (int i = 0; i < M && ok; ++i)
                ok = solve_row(M, i, t_host + (size_t)i * M, d.data() + (size_t)i * M, lb.data() + (size_t)i * M,
                               M * tbar, P.data() + (size_t)i * M, scratch);
            if (!ok) continue;
            // p_i of Eq. (d4)
            double fsum = 0.0;
            for (int i = 0; i < M; ++i) {
                double ti = 0.0;
                for (int m = 0; m < M; ++m)
                    if (d[(size_t)i * M + m]) ti += t_host[(size_t)i * M + m] * P[(size_t)i * M + m];
                act[i] = 1.0 / ti;
                fsum += act[i];
            }
            if (!std::isfinite(fsum)) continue;
            for (int i = 0; i < M; ++i) act[i] /= fsum;
            // Y_P, Eq. (d2)
            for (int i = 0; i < M; ++i)
                for (int m = 0; m < M; ++m) {
                    const size_t e = (size_t)i * M + m;
                    double gam = 0.0;
                    if (i != m && d[e] && P[e] > 0.0) gam = (d[e] + d[(size_t)m * M + i]) / (2.0 * P[e]);
                    a1[e] = act[i] * P[e] * gam;
                    a2[e] = act[i] * P[e] * gam * gam;
                }
            const double ar = alpha * rho;
            for (int i = 0; i < M; ++i) {
                double s1 = 0.0, s2 = 0.0;
                for (int m = 0; m < M; ++m) {
                    if (m == i) continue;
                    const size_t e = (size_t)i * M + m, f = (size_t)m * M + i;
                    Y[e] = ar * (a1[e] + a1[f]) - ar * ar * (a2[e] + a2[f]);
                    s1 += a1[e];
                    s2 += a2[e] + a2[f];
                }
                Y[(size_t)i * M + i] = 1.0 - 2.0 * ar * s1 + ar * ar * s2;
            }
            for (int i = 0; i < M; ++i)      // symmetrise against rounding
                for (int m = i + 1; m < M; ++m) {
                    const double v = 0.5 * (Y[(size_t)i * M + m] + Y[(size_t)m * M + i]);
                    Y[(size_t)i * M + m] = Y[(size_t)m * M + i] = v;
                }
            symmetric_eigenvalues(M, Y, ev);
            const double lam2 = ev[M - 2];
            if (!(lam2 > 0.0) || !(lam2 < 1.0)) continue;
            const double conv = tbar * std::log(eps) / std::log(lam2);
            if (!found || conv < best_conv) {
                found = true;
                best_conv = conv;
                best_P = P;
                *rho_out = rho;
                if (tbar_out) *tbar_out = tbar;
                if (lambda2_out) *lambda2_out = lam2;
                if (t_conv_out) *t_conv_out = conv;
            }
        }
    }
    if (!found) return NETMAX_EINFEASIBLE;
    std::copy(best_P.begin(), best_P.end(), P_out);
    return NETMAX_OK;
}
