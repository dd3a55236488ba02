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
//
// A second route (further down) reaches the same vector from a factor of the whole
// matrix computed once per layer, at a cost that grows with the number of stragglers
// instead of the number of responders.
#include <algorithm>
#include <cmath>
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

namespace {

// Householder QR with column pivoting of the m x c matrix M (column-major, leading dimension
// m, columns at most NGC_MAX_N long), in place, stopped at the numerical rank, which is
// returned.  On return column j < rank holds R[0..j][j] above the diagonal and the reflector's
// tail below it; piv[j] is the original index of the column now in position j.
int qr_pivoted(double* M, int m, int c, int* piv, double* tau) {
    for (int j = 0; j < c; ++j) piv[j] = j;
    // squared norms of the not yet eliminated part of every column; downdated after each
    // reflection and recomputed when cancellation has eaten most of the digits
    double cn[NGC_MAX_N], cn_ref[NGC_MAX_N];
    for (int j = 0; j < c; ++j) {
        const double* col = &M[(size_t)j * m];
        cn[j] = cn_ref[j] = dot4(col, col, m);
    }
    double norm0 = 0.0;
    const int kmax = std::min(m, c);
    int rank = 0;
    for (int k = 0; k < kmax; ++k) {
        tau[k] = 0.0;
        int best = k;
        double bestn = -1.0;
        for (int j = k; j < c; ++j)
            if (cn[j] > bestn) { bestn = cn[j]; best = j; }
        {   // the pivot's norm is always taken from the data itself
            const double* col = &M[(size_t)best * m];
            bestn = std::sqrt(dot4(col + k, col + k, m - k));
        }
        if (k == 0) norm0 = bestn;
        if (!(bestn > 1e-11 * norm0) || bestn == 0.0) {
            // the downdated norms may have drifted: look again with exact norms before stopping
            bestn = -1.0;
            for (int j = k; j < c; ++j) {
                const double* col = &M[(size_t)j * m];
                const double sq = dot4(col + k, col + k, m - k);
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
            for (int i = 0; i < m; ++i) std::swap(M[(size_t)best * m + i], M[(size_t)k * m + i]);
        }
        // Householder reflector H = I - tau v v^T, v[k] = 1, zeroing M[k+1:, k]
        double* col = &M[(size_t)k * m];
        double alpha = col[k];
        const double xn = dot4(col + k + 1, col + k + 1, m - k - 1);
        if (xn != 0.0) {
            double beta = -std::copysign(std::sqrt(alpha * alpha + xn), alpha);
            tau[k] = (beta - alpha) / beta;
            double scale = 1.0 / (alpha - beta);
            for (int i = k + 1; i < m; ++i) col[i] *= scale;
            col[k] = beta;
            for (int j = k + 1; j < c; ++j) {
                double* cj = &M[(size_t)j * m];
                double w = (cj[k] + dot4(col + k + 1, cj + k + 1, m - k - 1)) * tau[k];
                cj[k] -= w;
                for (int i = k + 1; i < m; ++i) cj[i] -= w * col[i];
            }
        }
        for (int j = k + 1; j < c; ++j) {
            const double rkj = M[(size_t)j * m + k];
            cn[j] -= rkj * rkj;
            if (!(cn[j] > 1e-4 * cn_ref[j])) {  // too much cancellation: recompute
                const double* cj = &M[(size_t)j * m];
                cn[j] = cn_ref[j] = dot4(cj + k + 1, cj + k + 1, m - k - 1);
            }
        }
        rank = k + 1;
    }
    return rank;
}

// x <- H_0 H_1 ... H_{rank-1} x for the reflectors left in M by qr_pivoted
void apply_q(const double* M, int m, int rank, const double* tau, double* x) {
    for (int k = rank - 1; k >= 0; --k) {
        if (tau[k] == 0.0) continue;
        const double* col = &M[(size_t)k * m];
        double w = x[k];
        for (int i = k + 1; i < m; ++i) w += col[i] * x[i];
        w *= tau[k];
        x[k] -= w;
        for (int i = k + 1; i < m; ++i) x[i] -= w * col[i];
    }
}

// Least-norm x (m entries) with (column piv[j])^T x = rhs[piv[j]] for the rank pivot columns:
// R11^T z = rhs (lower triangular, forward substitution), x = Q [z; 0].
void min_norm_from_qr(const double* M, int m, int rank, const int* piv, const double* tau,
                      const double* rhs, double* x) {
    for (int i = 0; i < m; ++i) x[i] = 0.0;
    for (int j = 0; j < rank; ++j) {
        double acc = rhs[piv[j]];
        for (int i = 0; i < j; ++i) acc -= M[(size_t)j * m + i] * x[i];
        x[j] = acc / M[(size_t)j * m + j];
    }
    apply_q(M, m, rank, tau, x);
}

double decode_residual(const double* B, int n, const int* rows, int ns, const double* a) {
    double acc[NGC_MAX_N];
    for (int j = 0; j < n; ++j) acc[j] = 0.0;
    for (int i = 0; i < ns; ++i) {
        const double ai = a[rows[i]];
        const double* b = &B[(size_t)rows[i] * n];
        for (int j = 0; j < n; ++j) acc[j] += ai * b[j];
    }
    double worst = 0.0;
    for (int j = 0; j < n; ++j) worst = std::max(worst, std::fabs(acc[j] - 1.0));
    return worst;
}

}  // namespace

int ngc_min_norm_decode(const double* B, int nw, int n, const int* rows, int ns, double* a_out,
                        double* resid) {
    // nw workers (length of a), n = k columns of B
    for (int i = 0; i < nw; ++i) a_out[i] = 0.0;
    if (ns <= 0) {
        if (resid) *resid = 1.0;
        return 0;
    }
    // M: ns x n, column-major (column j contiguous), M[:,j] = B[rows, j]
    double M[NGC_MAX_N * NGC_MAX_N];
    for (int j = 0; j < n; ++j)
        for (int i = 0; i < ns; ++i) M[(size_t)j * ns + i] = B[(size_t)rows[i] * n + j];
    int piv[NGC_MAX_N];
    double tau[NGC_MAX_N], ones[NGC_MAX_N], z[NGC_MAX_N];
    const int rank = qr_pivoted(M, ns, n, piv, tau);
    for (int j = 0; j < n; ++j) ones[j] = 1.0;
    min_norm_from_qr(M, ns, rank, piv, tau, ones, z);
    for (int i = 0; i < ns; ++i) a_out[rows[i]] = z[i];
    if (resid) *resid = decode_residual(B, n, rows, ns, a_out);
    return rank;
}

// ---------------------------------------------------------------------------
// The same decode vector by way of the full-response solution.
//
// Let a0 be the least-norm solution when every worker responds, and let the columns of N
// (nw x q, orthonormal) span {v : v^T B = 0}.  Every solution of a^T B = 1^T is a0 + N w,
// and a0 is orthogonal to N, so |a|^2 = |a0|^2 + |w|^2: the least-norm solution that vanishes
// on the stragglers T is a0 + N w with w the least-norm solution of N_T w = -a0_T, a system
// with one equation per straggler and q unknowns.  For a cyclic code q equals the layer's
// tolerance, so this costs about q |T|^2 operations instead of the n k (n - |T|) of the
// factorisation above.
// ---------------------------------------------------------------------------
int ngc_null_factor(const double* B, int nw, int n, double* a0, double* N, double* resid) {
    int all[NGC_MAX_N];
    for (int i = 0; i < nw; ++i) all[i] = i;
    double M[NGC_MAX_N * NGC_MAX_N];
    for (int j = 0; j < n; ++j)
        for (int i = 0; i < nw; ++i) M[(size_t)j * nw + i] = B[(size_t)i * n + j];
    int piv[NGC_MAX_N];
    double tau[NGC_MAX_N], ones[NGC_MAX_N];
    const int rank = qr_pivoted(M, nw, n, piv, tau);
    for (int j = 0; j < n; ++j) ones[j] = 1.0;
    min_norm_from_qr(M, nw, rank, piv, tau, ones, a0);
    if (resid) *resid = decode_residual(B, n, all, nw, a0);
    // the last nw - rank columns of Q are orthogonal to every column of B
    const int q = nw - rank;
    double e[NGC_MAX_N];
    for (int t = 0; t < q; ++t) {
        for (int i = 0; i < nw; ++i) e[i] = 0.0;
        e[rank + t] = 1.0;
        apply_q(M, nw, rank, tau, e);
        for (int i = 0; i < nw; ++i) N[(size_t)i * q + t] = e[i];  // row i of N is contiguous
    }
    return q;
}

int ngc_min_norm_decode_null(const double* B, int nw, int n, const double* a0, const double* N,
                             int q, const int* rows, int ns, double* a_out, double* resid) {
    for (int i = 0; i < nw; ++i) a_out[i] = 0.0;
    if (ns <= 0) {
        if (resid) *resid = 1.0;
        return 0;
    }
    // stragglers: the workers not listed in rows (rows ascending)
    int T[NGC_MAX_N];
    int nt = 0;
    for (int i = 0, r = 0; i < nw; ++i) {
        if (r < ns && rows[r] == i) ++r;
        else T[nt++] = i;
    }
    double w[NGC_MAX_N];
    int rank = 0;
    if (nt > 0 && q > 0) {
        // columns of M (q x nt): the stragglers' rows of N
        double M[NGC_MAX_N * NGC_MAX_N];
        double rhs[NGC_MAX_N], tau[NGC_MAX_N];
        int piv[NGC_MAX_N];
        for (int t = 0; t < nt; ++t) {
            const double* src = &N[(size_t)T[t] * q];
            for (int i = 0; i < q; ++i) M[(size_t)t * q + i] = src[i];
            rhs[t] = -a0[T[t]];
        }
        rank = qr_pivoted(M, q, nt, piv, tau);
        min_norm_from_qr(M, q, rank, piv, tau, rhs, w);
    } else {
        for (int i = 0; i < q; ++i) w[i] = 0.0;
    }
    for (int r = 0; r < ns; ++r) {
        const int i = rows[r];
        a_out[i] = a0[i] + dot4(&N[(size_t)i * q], w, q);
    }
    if (resid) *resid = decode_residual(B, n, rows, ns, a_out);
    return rank;
}
