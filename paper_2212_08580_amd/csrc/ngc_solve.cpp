// Decode-vector selection on the host (Def. 1 of the paper, last two bullets):
// find a, supported on the responders S, with a^T B = 1^T.  Among all solutions
// the one of least 2-norm is returned; it lies in the column space of B_S
// (n_S x n), so a = Q z where Q is an orthonormal basis of that space.
//
// Method: Householder QR of B_S with column pivoting, stopped at the numerical
// rank r.  The r pivot columns give r independent equations
//   (Q R11)^T a = 1   =>   R11^T z = 1,   a = Q [z; 0].
// The remaining n - r equations are linear combinations of these because the
// system is consistent whenever B is a gradient code and |S| >= n - sigma; the
// caller checks the residual over all k columns.  fp64 throughout, n, k <= 64.
#include <algorithm>
#include <cmath>
#include <vector>

#include "ngc_internal.h"

// dot product with four running sums (lets the compiler use 4-wide vectors without
// being allowed to reassociate a single sum)
static inline double dot4(const double* __restrict__ x, const double* __restrict__ y, int len) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int i = 0;
    for (; i + 4 <= len; i += 4) {
        s0 += x[i] * y[i];
        s1 += x[i + 1] * y[i + 1];
        s2 += x[i + 2] * y[i + 2];
        s3 += x[i + 3] * y[i + 3];
    }
    for (; i < len; ++i) s0 += x[i] * y[i];
    return (s0 + s1) + (s2 + s3);
}

int ngc_min_norm_decode(const double* B, int nw, int n, const int* rows, int ns, double* a_out,
                        double* resid) {
    // nw workers (length of a), n = k columns of B
    for (int i = 0; i < nw; ++i) a_out[i] = 0.0;
    if (ns <= 0) {
        if (resid) *resid = 1.0;
        return 0;
    }
    // M: ns x n, column-major (column j contiguous), M[:,j] = B[rows, j]
    std::vector<double> M((size_t)ns * n);
    for (int j = 0; j < n; ++j)
        for (int i = 0; i < ns; ++i) M[(size_t)j * ns + i] = B[(size_t)rows[i] * n + j];
    std::vector<int> piv(n);
    for (int j = 0; j < n; ++j) piv[j] = j;
    std::vector<double> tau(std::min(ns, n), 0.0);

    // squared norms of the not yet eliminated part of every column; downdated after each
    // reflection and recomputed when cancellation has eaten most of the digits
    std::vector<double> cn(n), cn_ref(n);
    for (int j = 0; j < n; ++j) {
        const double* c = &M[(size_t)j * ns];
        cn[j] = cn_ref[j] = dot4(c, c, ns);
    }
    double norm0 = 0.0;
    const int kmax = std::min(ns, n);
    int rank = 0;
    for (int k = 0; k < kmax; ++k) {
        int best = k;
        double bestn = -1.0;
        for (int j = k; j < n; ++j)
            if (cn[j] > bestn) { bestn = cn[j]; best = j; }
        {   // the pivot's norm is always taken from the data itself
            const double* c = &M[(size_t)best * ns];
            bestn = std::sqrt(dot4(c + k, c + k, ns - k));
        }
        if (k == 0) norm0 = bestn;
        if (!(bestn > 1e-11 * norm0) || bestn == 0.0) {
            // the downdated norms may have drifted: look again with exact norms before stopping
            bestn = -1.0;
            for (int j = k; j < n; ++j) {
                const double* c = &M[(size_t)j * ns];
                const double sq = dot4(c + k, c + k, ns - k);
                cn[j] = cn_ref[j] = sq;
                if (sq > bestn) { bestn = sq; best = j; }
            }
            bestn = std::sqrt(bestn);
            if (!(bestn > 1e-11 * norm0) || bestn == 0.0) break;
        }
        if (best != k) {
            std::swap(piv[best], piv[k]);
            std::swap(cn[best], cn[k]);
            std::swap(cn_ref[best], cn_ref[k]);
            for (int i = 0; i < ns; ++i) std::swap(M[(size_t)best * ns + i], M[(size_t)k * ns + i]);
        }
        // Householder reflector H = I - tau v v^T, v[k] = 1, zeroing M[k+1:, k]
        double* c = &M[(size_t)k * ns];
        double alpha = c[k];
        const double xn = dot4(c + k + 1, c + k + 1, ns - k - 1);
        if (xn == 0.0) {
            tau[k] = 0.0;
        } else {
            double beta = -std::copysign(std::sqrt(alpha * alpha + xn), alpha);
            tau[k] = (beta - alpha) / beta;
            double scale = 1.0 / (alpha - beta);
            for (int i = k + 1; i < ns; ++i) c[i] *= scale;
            c[k] = beta;
            for (int j = k + 1; j < n; ++j) {
                double* cj = &M[(size_t)j * ns];
                double w = (cj[k] + dot4(c + k + 1, cj + k + 1, ns - k - 1)) * tau[k];
                cj[k] -= w;
                for (int i = k + 1; i < ns; ++i) cj[i] -= w * c[i];
            }
        }
        for (int j = k + 1; j < n; ++j) {
            const double rkj = M[(size_t)j * ns + k];
            cn[j] -= rkj * rkj;
            if (!(cn[j] > 1e-4 * cn_ref[j])) {  // too much cancellation: recompute
                const double* cj = &M[(size_t)j * ns];
                cn[j] = cn_ref[j] = dot4(cj + k + 1, cj + k + 1, ns - k - 1);
            }
        }
        rank = k + 1;
    }
    // forward substitution with R11^T (lower triangular): sum_{i<=j} R[i][j] z[i] = 1
    std::vector<double> z(ns, 0.0);
    for (int j = 0; j < rank; ++j) {
        double acc = 1.0;
        for (int i = 0; i < j; ++i) acc -= M[(size_t)j * ns + i] * z[i];
        z[j] = acc / M[(size_t)j * ns + j];
    }
    // a_S = H_0 H_1 ... H_{r-1} [z; 0]
    for (int k = rank - 1; k >= 0; --k) {
        if (tau[k] == 0.0) continue;
        const double* c = &M[(size_t)k * ns];
        double w = z[k];
        for (int i = k + 1; i < ns; ++i) w += c[i] * z[i];
        w *= tau[k];
        z[k] -= w;
        for (int i = k + 1; i < ns; ++i) z[i] -= w * c[i];
    }
    for (int i = 0; i < ns; ++i) a_out[rows[i]] = z[i];
    if (resid) {
        double worst = 0.0;
        for (int j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int i = 0; i < ns; ++i) acc += z[i] * B[(size_t)rows[i] * n + j];
            worst = std::max(worst, std::fabs(acc - 1.0));
        }
        *resid = worst;
    }
    return rank;
}
