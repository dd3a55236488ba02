// Latency model of Secs. II-D and IV, closed forms on the host: the CDF of the time a
// conventional (n,k,sigma) gradient code needs (Lemma 1) and of a nested code (Theorem 1).
//
// A non-failing worker finishes u tasks at gamma + eps + u*rho + Erlang(u, lambda);
// a worker fails for good with probability p_e.  A conventional code with
// tolerance sigma is done when n - sigma workers have finished sigma + 1 tasks,
// a nested code when any of its component codes sigma = 0..s_max is.
//
// Readings: the Erlang CDF sums to u-1 (eq. (3) prints u; the identity in the
// proof of Corollary 1 needs u-1); the summation limits of Theorem 1 follow its
// proof (a configuration counts as "not decodable" when at every layer u fewer
// than n-u+1 workers have finished u tasks), not the limit printed in the
// statement, which lets decodable configurations through.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/ngc.h"

int ngc_on_exception();  // ngc_host.cpp: status for an exception caught at the C boundary

bool ngc_latency_bad_params(int n, int s, double lam, double rho, double eps, double gamma, double pe) {
    return n < 1 || n > 64 || s < 0 || s >= n || !(lam > 0.0) || !(rho >= 0.0) || !(eps >= 0.0) ||
           !(gamma >= 0.0) || !(pe >= 0.0) || !(pe <= 1.0);
}

namespace {

// F_u(t): P(gamma + eps + u rho + Erlang(u, lam) <= t)
double layer_cdf(int u, double t, double lam, double rho, double eps, double gamma) {
    const double tau = t - (gamma + eps + u * rho);
    if (tau < 0.0) return 0.0;
    if (u == 0) return 1.0;
    const double x = lam * tau;
    double term = 1.0, sum = 1.0;  // sum_{v<u} x^v / v!
    for (int v = 1; v < u; ++v) {
        term *= x / v;
        sum += term;
    }
    return 1.0 - std::exp(-x) * sum;
}

struct binomials {
    std::vector<double> c;
    int n;
    explicit binomials(int n_) : c((size_t)(n_ + 1) * (n_ + 1), 0.0), n(n_) {
        for (int a = 0; a <= n; ++a) {
            c[(size_t)a * (n + 1)] = 1.0;
            for (int b = 1; b <= a; ++b)
                c[(size_t)a * (n + 1) + b] = c[(size_t)(a - 1) * (n + 1) + b - 1] +
                                             (b <= a - 1 ? c[(size_t)(a - 1) * (n + 1) + b] : 0.0);
        }
    }
    double operator()(int a, int b) const { return (b < 0 || b > a) ? 0.0 : c[(size_t)a * (n + 1) + b]; }
};

}  // namespace

extern "C" int ngc_latency_cdf_gc(int n, int sigma, double lam, double rho, double eps, double gamma,
                                  double pe, const double* t, int nt, double* cdf_out) try {
    if (ngc_latency_bad_params(n, sigma, lam, rho, eps, gamma, pe) || !t || !cdf_out || nt < 0) return NGC_ERR_INVALID;
    binomials C(n);
    for (int q = 0; q < nt; ++q) {
        const double F = layer_cdf(sigma + 1, t[q], lam, rho, eps, gamma);
        double total = 0.0;
        for (int kappa = 0; kappa <= sigma; ++kappa) {
            const int alive = n - kappa;
            double cond = 0.0;
            for (int m = n - sigma; m <= alive; ++m)
                cond += C(alive, m) * std::pow(F, m) * std::pow(1.0 - F, alive - m);
            total += cond * C(n, kappa) * std::pow(pe, kappa) * std::pow(1.0 - pe, n - kappa);
        }
        cdf_out[q] = total;
    }
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_latency_cdf_ngc(int n, int smax, double lam, double rho, double eps, double gamma,
                                   double pe, const double* t, int nt, double* cdf_out) try {
    if (ngc_latency_bad_params(n, smax, lam, rho, eps, gamma, pe) || !t || !cdf_out || nt < 0) return NGC_ERR_INVALID;
    binomials C(n);
    const int top = smax + 1;
    std::vector<double> p(top + 2), g(n + 1), h(n + 1);
    for (int q = 0; q < nt; ++q) {
        std::vector<double> F(top + 2);
        for (int u = 0; u <= top + 1; ++u) F[u] = layer_cdf(u, t[q], lam, rho, eps, gamma);
        for (int u = 1; u < top; ++u) p[u] = F[u] - F[u + 1];   // finished exactly u tasks
        p[top] = F[top];                                        // finished all of them
        const double q0 = 1.0 - F[1];                           // finished none
        double total = 0.0;
        for (int kappa = 0; kappa <= smax; ++kappa) {
            const int alive = n - kappa;
            // g[S] = weight of all assignments of S workers to the layers above the current one
            // in which none of those layers has its n-u+1 finishers
            std::fill(g.begin(), g.end(), 0.0);
            g[0] = 1.0;
            for (int u = top; u >= 1; --u) {
                std::fill(h.begin(), h.end(), 0.0);
                const int cap = std::min(n - u, alive);  // at most n-u workers with >= u tasks
                for (int S = 0; S <= cap; ++S) {
                    if (g[S] == 0.0) continue;
                    double pw = 1.0;
                    for (int S2 = S; S2 <= cap; ++S2) {
                        h[S2] += g[S] * C(alive - S, S2 - S) * pw;
                        pw *= p[u];
                    }
                }
                g.swap(h);
            }
            double stuck = 0.0;
            for (int S = 0; S <= alive; ++S) stuck += g[S] * std::pow(q0, alive - S);
            total += (1.0 - stuck) * C(n, kappa) * std::pow(pe, kappa) * std::pow(1.0 - pe, n - kappa);
        }
        cdf_out[q] = total;
    }
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}
