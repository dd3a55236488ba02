// Host side of libngc: context life cycle, code tables (Sec. III, Defs. 1-2,
// Alg. 1, Lemma 2), layer choice and decode-vector selection.  No HIP call is
// made from this file.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "ngc_internal.h"

int ngc_fail(const ngc_ctx* ctx, int code, const std::string& msg) {
    if (ctx) ctx->err = msg;
    return code;
}

int ngc_on_exception() {
    try {
        throw;
    } catch (const std::bad_alloc&) {
        return NGC_ERR_NOMEM;
    } catch (...) {
        return NGC_ERR_INVALID;
    }
}

extern "C" const char* ngc_strerror(int code) {
    switch (code) {
        case NGC_OK: return "ok";
        case NGC_ERR_INVALID: return "invalid argument";
        case NGC_ERR_UNDECODABLE: return "more stragglers than the code tolerates";
        case NGC_ERR_SINGULAR: return "no decode vector: responders do not span the all-ones row";
        case NGC_ERR_HIP: return "HIP runtime error";
        case NGC_ERR_NOMEM: return "out of memory";
        case NGC_ERR_STATE: return "context not ready for this call";
        default: return "unknown error code";
    }
}

extern "C" const char* ngc_last_error(const ngc_ctx* ctx) { return ctx ? ctx->err.c_str() : ""; }

static void compress_layer(ngc_layer_code& lc, int n, int k) {
    lc.rowptr.assign(n + 1, 0);
    lc.col.clear();
    lc.coef.clear();
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j < k; ++j) {
            double v = lc.B[(size_t)i * k + j];
            if (v != 0.0) {
                lc.col.push_back(j);
                lc.coef.push_back(v);
            }
        }
        lc.rowptr[i + 1] = (int)lc.col.size();
    }
}

static void install_layer(ngc_ctx* ctx, int layer, const double* B) {
    ngc_layer_code& lc = ctx->code[layer];
    lc.A.clear();  // a decoding table belongs to the matrix it was built from
    lc.A_rows = 0;
    lc.A_stale = true;
    lc.B.assign(B, B + (size_t)ctx->n * ctx->k);
    compress_layer(lc, ctx->n, ctx->k);
    lc.row_norm.assign(ctx->n, 0.0);
    for (int i = 0; i < ctx->n; ++i) {
        double q = 0.0;
        for (int j = 0; j < ctx->k; ++j) q += B[(size_t)i * ctx->k + j] * B[(size_t)i * ctx->k + j];
        lc.row_norm[i] = std::sqrt(q);
    }
    lc.a0.assign(ctx->n, 0.0);
    lc.N.assign((size_t)ctx->n * ctx->n, 0.0);
    double full_resid = 1.0;
    lc.q = ngc_null_factor(lc.B.data(), ctx->n, ctx->k, lc.a0.data(), lc.N.data(), &full_resid);
    lc.null_ok = full_resid <= 1e-9;
    lc.set = true;
    ctx->code_dirty = true;
    ctx->wtab_dirty = true;
}

extern "C" int ngc_create(ngc_ctx** out, int n, int k, int L, const int* s, int64_t d,
                          void* hip_stream) try {
    if (!out) return NGC_ERR_INVALID;
    *out = nullptr;
    if (n < 1 || n > NGC_MAX_N || k < n || k > NGC_MAX_N || k % n != 0 || L < 1 || L > NGC_MAX_N ||
        !s || d < 1)
        return NGC_ERR_INVALID;
    if (s[0] != 0) return NGC_ERR_INVALID;
    for (int u = 1; u < L; ++u)
        if (s[u] <= s[u - 1]) return NGC_ERR_INVALID;
    if (s[L - 1] >= n) return NGC_ERR_INVALID;
    // 2^33 floats are 32 GiB per gradient row; beyond that the column-tile counts of the
    // kernels' grids would no longer fit their 31 bits
    if (d > ((int64_t)1 << 33)) return NGC_ERR_INVALID;
    ngc_ctx* ctx = new (std::nothrow) ngc_ctx;
    if (!ctx) return NGC_ERR_NOMEM;
    ctx->n = n;
    ctx->k = k;
    ctx->c = k / n;
    ctx->L = L;
    ctx->d = d;
    ctx->s.assign(s, s + L);
    ctx->stream = (hipStream_t)hip_stream;
    ctx->code.resize(L);
    // Alg. 1: B_0 = I; with c partitions per atomic task worker i holds group i: I (x) 1_{1 x c}
    std::vector<double> I((size_t)n * k, 0.0);
    for (int i = 0; i < n; ++i)
        for (int q = 0; q < ctx->c; ++q) I[(size_t)i * k + i * ctx->c + q] = 1.0;
    install_layer(ctx, 0, I.data());
    *out = ctx;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" void ngc_destroy(ngc_ctx* ctx) {
    if (!ctx) return;
    ngc_dev_release(ctx);
    delete ctx;
}

extern "C" int ngc_set_code(ngc_ctx* ctx, int layer, const double* B_host) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->L || !B_host) return ngc_fail(ctx, NGC_ERR_INVALID, "bad layer or null B");
    const int n = ctx->n, k = ctx->k, c = ctx->c;
    for (size_t t = 0; t < (size_t)n * k; ++t)
        if (!std::isfinite(B_host[t])) return ngc_fail(ctx, NGC_ERR_INVALID, "B has a non-finite entry");
    for (int i = 0; i < n; ++i) {
        for (int q = 0; q < c; ++q)
            if (B_host[(size_t)i * k + i * c + q] == 0.0)
                return ngc_fail(ctx, NGC_ERR_INVALID, "worker i must hold its own partition(s) (B[i][i*c..] != 0)");
        // Def. 2: supports grow with the layer
        for (int j = 0; j < k; ++j) {
            bool here = B_host[(size_t)i * k + j] != 0.0;
            for (int v = 0; v < ctx->L; ++v) {
                if (v == layer || !ctx->code[v].set) continue;
                bool there = ctx->code[v].B[(size_t)i * k + j] != 0.0;
                if (v < layer && there && !here)
                    return ngc_fail(ctx, NGC_ERR_INVALID, "row support does not contain the layer below (Def. 2)");
                if (v > layer && here && !there)
                    return ngc_fail(ctx, NGC_ERR_INVALID, "row support is not contained in the layer above (Def. 2)");
            }
        }
    }
    install_layer(ctx, layer, B_host);
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_get_code(const ngc_ctx* ctx, int layer, double* B_host_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->L || !B_host_out) return ngc_fail(ctx, NGC_ERR_INVALID, "bad layer or null output");
    if (!ctx->code[layer].set) return ngc_fail(ctx, NGC_ERR_STATE, "layer has no code yet");
    std::memcpy(B_host_out, ctx->code[layer].B.data(), sizeof(double) * ctx->n * ctx->k);
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_get_shape(const ngc_ctx* ctx, int* n_out, int* k_out, int* layers_out, int64_t* d_out,
                             int* mlp_d_in_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (n_out) *n_out = ctx->n;
    if (k_out) *k_out = ctx->k;
    if (layers_out) *layers_out = ctx->L;
    if (d_out) *d_out = ctx->d;
    if (mlp_d_in_out) *mlp_d_in_out = ctx->mlp_din;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_set_mlp2_shape(ngc_ctx* ctx, int d_in, int hidden, int classes) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (d_in < 1 || hidden < 1 || classes < 2) return ngc_fail(ctx, NGC_ERR_INVALID, "bad MLP shape");
    int64_t need = (int64_t)d_in * hidden + hidden + (int64_t)hidden * classes + classes;
    if (need != ctx->d) return ngc_fail(ctx, NGC_ERR_INVALID, "MLP parameter count differs from d");
    ctx->mlp_din = d_in;
    ctx->mlp_hidden = hidden;
    ctx->mlp_classes = classes;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---------------------------------------------------------------------------
// Random numbers for the code construction: Philox-4x32 with 10 rounds
// (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC'11), a counter-based generator: output = bijection_key(counter).
// ---------------------------------------------------------------------------
namespace {

struct Philox {
    uint32_t key[2];
    uint64_t ctr_lo = 0, ctr_hi;
    uint32_t out[4];
    int have = 0;
    Philox(uint64_t seed, uint64_t stream) : ctr_hi(stream) {
        key[0] = (uint32_t)seed;
        key[1] = (uint32_t)(seed >> 32);
    }
    void block() {
        uint32_t c[4] = {(uint32_t)ctr_lo, (uint32_t)(ctr_lo >> 32), (uint32_t)ctr_hi, (uint32_t)(ctr_hi >> 32)};
        uint32_t k0 = key[0], k1 = key[1];
        for (int r = 0; r < 10; ++r) {
            uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
            uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
            uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
            uint32_t n1 = (uint32_t)p1;
            uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
            uint32_t n3 = (uint32_t)p0;
            c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        std::memcpy(out, c, sizeof(out));
        ++ctr_lo;
        have = 4;
    }
    uint32_t u32() {
        if (!have) block();
        return out[4 - have--];
    }
    double uniform() {  // (0,1], 53 bits
        uint64_t hi = u32(), lo = u32();
        uint64_t x = ((hi << 32) | lo) >> 11;
        return ((double)x + 1.0) * (1.0 / 9007199254740992.0);
    }
    double normal() {  // Box-Muller, one value per call
        double u1 = uniform(), u2 = uniform();
        return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
    }
    int below(int m) { return (int)(((uint64_t)u32() * (uint64_t)m) >> 32); }
};

// Solve the s x s system A x = b in place by Gaussian elimination with partial
// pivoting.  A row-major.  Returns false if a pivot vanishes.
bool solve_square(std::vector<double>& A, std::vector<double>& b, int s) {
    for (int c = 0; c < s; ++c) {
        int p = c;
        for (int r = c + 1; r < s; ++r)
            if (std::fabs(A[(size_t)r * s + c]) > std::fabs(A[(size_t)p * s + c])) p = r;
        if (A[(size_t)p * s + c] == 0.0) return false;
        if (p != c) {
            for (int j = 0; j < s; ++j) std::swap(A[(size_t)p * s + j], A[(size_t)c * s + j]);
            std::swap(b[p], b[c]);
        }
        for (int r = c + 1; r < s; ++r) {
            double f = A[(size_t)r * s + c] / A[(size_t)c * s + c];
            if (f == 0.0) continue;
            for (int j = c; j < s; ++j) A[(size_t)r * s + j] -= f * A[(size_t)c * s + j];
            b[r] -= f * b[c];
        }
    }
    for (int r = s - 1; r >= 0; --r) {
        double acc = b[r];
        for (int j = r + 1; j < s; ++j) acc -= A[(size_t)r * s + j] * b[j];
        b[r] = acc / A[(size_t)r * s + r];
    }
    return true;
}

// One random cyclic code with tolerance sigma: rows in the null space of H
// (sigma x n, Gaussian, rows summing to zero), row i supported on {i..i+sigma}.
bool draw_cyclic(int n, int sigma, Philox& rng, std::vector<double>& B) {
    std::vector<double> H((size_t)sigma * n);
    for (int r = 0; r < sigma; ++r) {
        double sum = 0.0;
        for (int j = 0; j < n - 1; ++j) {
            H[(size_t)r * n + j] = rng.normal();
            sum += H[(size_t)r * n + j];
        }
        H[(size_t)r * n + n - 1] = -sum;
    }
    B.assign((size_t)n * n, 0.0);
    std::vector<double> A((size_t)sigma * sigma), rhs(sigma);
    for (int i = 0; i < n; ++i) {
        for (int r = 0; r < sigma; ++r) {
            for (int t = 1; t <= sigma; ++t) A[(size_t)r * sigma + t - 1] = H[(size_t)r * n + (i + t) % n];
            rhs[r] = -H[(size_t)r * n + i];
        }
        if (!solve_square(A, rhs, sigma)) return false;
        B[(size_t)i * n + i] = 1.0;
        for (int t = 1; t <= sigma; ++t) B[(size_t)i * n + (i + t) % n] = rhs[t - 1];
    }
    return true;
}

// How much decoding magnifies rounding of the messages when exactly sigma workers straggle (then
// the decode vector is the only one there is): sum_i |a_i| ||b_i||_2, the factor between the
// relative rounding of a message and the error of the decoded sum for partial gradients of
// equal size.  Score of a candidate code = the upper tail of that figure over straggler sets of
// size sigma: its maximum over all C(n, sigma) sets when there are at most `exhaustive` of them,
// else its ninth decile over `samples` random sets.  Infinite if a set cannot be decoded.
double amplification(const std::vector<double>& B, int n, int sigma, uint64_t seed, int samples,
                     int exhaustive) {
    std::vector<double> l2(n, 0.0), a(n), a0(n), N((size_t)n * n);
    for (int i = 0; i < n; ++i) {
        double sq = 0.0;
        for (int j = 0; j < n; ++j) sq += B[(size_t)i * n + j] * B[(size_t)i * n + j];
        l2[i] = std::sqrt(sq);
    }
    double full_resid = 1.0;
    const int q = ngc_null_factor(B.data(), n, n, a0.data(), N.data(), &full_resid);
    const bool null_ok = full_resid <= 1e-9;
    std::vector<int> rows;
    auto one = [&](const std::vector<char>& out) -> double {
        rows.clear();
        for (int i = 0; i < n; ++i)
            if (!out[i]) rows.push_back(i);
        double resid = 0.0;
        if (null_ok)
            ngc_min_norm_decode_null(B.data(), n, n, a0.data(), N.data(), q, rows.data(), (int)rows.size(), a.data(), &resid);
        else
            ngc_min_norm_decode(B.data(), n, n, rows.data(), (int)rows.size(), a.data(), &resid);
        if (!(resid < 1e-6)) return INFINITY;
        double tot = 0.0;
        for (int i = 0; i < n; ++i) tot += std::fabs(a[i]) * l2[i];
        return tot;
    };
    // number of straggler sets, saturating
    double count = 1.0;
    for (int t = 1; t <= sigma; ++t) count = count * (n - sigma + t) / t;
    std::vector<char> out(n, 0);
    if (count <= (double)exhaustive) {
        std::vector<int> c(sigma);
        for (int t = 0; t < sigma; ++t) c[t] = t;
        double worst = 0.0;
        for (;;) {
            std::fill(out.begin(), out.end(), 0);
            for (int t = 0; t < sigma; ++t) out[c[t]] = 1;
            worst = std::max(worst, one(out));
            if (!(worst < INFINITY)) return INFINITY;
            int j = sigma - 1;
            while (j >= 0 && c[j] == n - sigma + j) --j;
            if (j < 0) break;
            ++c[j];
            for (int t = j + 1; t < sigma; ++t) c[t] = c[t - 1] + 1;
        }
        return worst;
    }
    Philox rng(seed, 0x5c0feULL);
    std::vector<int> perm(n);
    std::vector<double> seen;
    for (int t = 0; t < samples; ++t) {
        for (int i = 0; i < n; ++i) perm[i] = i;
        for (int i = 0; i < sigma; ++i) std::swap(perm[i], perm[i + rng.below(n - i)]);
        std::fill(out.begin(), out.end(), 0);
        for (int i = 0; i < sigma; ++i) out[perm[i]] = 1;
        const double v = one(out);
        if (!(v < INFINITY)) return INFINITY;
        seen.push_back(v);
    }
    std::sort(seen.begin(), seen.end());
    return seen[std::min<size_t>(seen.size() - 1, (seen.size() * 9) / 10)];
}

}  // namespace

extern "C" int ngc_build_code(ngc_ctx* ctx, int kind, uint64_t seed) try {
    if (!ctx) return NGC_ERR_INVALID;
    const int n = ctx->n;
    if (kind != NGC_CODE_CYCLIC && kind != NGC_CODE_FRACREP) return ngc_fail(ctx, NGC_ERR_INVALID, "unknown code kind");
    std::vector<std::vector<double>> built(ctx->L);
    for (int u = 0; u < ctx->L; ++u) {
        const int sigma = ctx->s[u];
        std::vector<double>& B = built[u];
        if (sigma == 0) {
            B.assign((size_t)n * n, 0.0);
            for (int i = 0; i < n; ++i) B[(size_t)i * n + i] = 1.0;
        } else if (kind == NGC_CODE_FRACREP) {
            const int w = sigma + 1;
            if (n % w) return ngc_fail(ctx, NGC_ERR_INVALID, "fractional repetition needs (s+1) | n");
            if (w % (ctx->s[u - 1] + 1)) return ngc_fail(ctx, NGC_ERR_INVALID, "fractional-repetition layers are not nested");
            B.assign((size_t)n * n, 0.0);
            for (int i = 0; i < n; ++i)
                for (int j = w * (i / w); j < w * (i / w) + w; ++j) B[(size_t)i * n + j] = 1.0;
        } else {
            // the candidates are scored on the same straggler sets; the one whose decoding
            // magnifies message rounding least at full straggler count is kept
            const int draws = 48;
            double best = INFINITY;
            std::vector<double> cand;
            for (int t = 0; t < draws; ++t) {
                Philox rng(seed, ((uint64_t)sigma << 32) | (uint64_t)t);
                if (!draw_cyclic(n, sigma, rng, cand)) continue;
                double score = amplification(cand, n, sigma, seed ^ (uint64_t)sigma, 96, 6000);
                if (score < best) {
                    best = score;
                    B = cand;
                }
            }
            if (!(best < INFINITY)) return ngc_fail(ctx, NGC_ERR_SINGULAR, "no valid cyclic draw found");
        }
    }
    // k = c n partitions: worker i treats the c partitions of group j like partition j, B' (x) 1_{1 x c}
    const int k = ctx->k, c = ctx->c;
    std::vector<double> wide((size_t)n * k);
    for (int u = 0; u < ctx->L; ++u) ctx->code[u].set = false;
    for (int u = 0; u < ctx->L; ++u) {
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < k; ++j) wide[(size_t)i * k + j] = built[u][(size_t)i * n + j / c];
        install_layer(ctx, u, wide.data());
    }
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

void ngc_layer_decode_vec(const ngc_ctx* ctx, int layer, const int* rows, int ns, double* a_out,
                          double* resid) {
    const ngc_layer_code& lc = ctx->code[layer];
    const int n = ctx->n, k = ctx->k;
    const int nt = n - ns, rank = n - lc.q;
    // operation counts of the two factorisations: n_S x k to rank `rank` against q x |T|
    const long direct = (long)ns * k * std::min(ns, rank);
    const long via_null = (long)lc.q * nt * nt + (long)ns * lc.q;
    if (lc.null_ok && via_null < direct)
        ngc_min_norm_decode_null(lc.B.data(), n, k, lc.a0.data(), lc.N.data(), lc.q, rows, ns, a_out, resid);
    else
        ngc_min_norm_decode(lc.B.data(), n, k, rows, ns, a_out, resid);
}

int ngc_select_core(const ngc_ctx* ctx, const uint8_t* mask, int* layer_out, double* a_out,
                    double* residual_out, bool first_only) {
    const int n = ctx->n;
    int stragglers = 0;
    for (int i = 0; i < n; ++i) stragglers += mask[i] != 0;
    for (int i = 0; i < n; ++i) a_out[i] = 0.0;
    int u = -1;
    for (int v = 0; v < ctx->L; ++v)
        if (ctx->s[v] >= stragglers) { u = v; break; }
    *layer_out = u;
    if (residual_out) *residual_out = 0.0;
    if (u < 0) return NGC_ERR_UNDECODABLE;
    if (!ctx->code[u].set) return NGC_ERR_STATE;
    int rows[NGC_MAX_N];
    int ns = 0;
    const int want = first_only ? n - ctx->s[u] : n;
    for (int i = 0; i < n && ns < want; ++i)
        if (!mask[i]) rows[ns++] = i;
    double resid = 0.0;
    ngc_layer_decode_vec(ctx, u, rows, ns, a_out, &resid);
    if (residual_out) *residual_out = resid;
    if (!(resid <= 1e-6)) return NGC_ERR_SINGULAR;
    // Guarded choice (off unless a limit is set): every component code with s_v >= #stragglers
    // recovers the gradient (Def. 1); if the estimated amplification of message rounding at the
    // smallest such layer exceeds the limit, the first layer above it within the limit is
    // taken, else the layer of smallest estimate (the lowest on a tie).
    if (!first_only && ctx->guard_limit > 0.0) {
        auto kappa_hat = [&](int v, const double* a) {
            double q = 0.0;
            for (int i = 0; i < n; ++i) q += std::fabs(a[i]) * ctx->code[v].row_norm[i];
            return q / std::sqrt((double)ctx->k);
        };
        double best = kappa_hat(u, a_out);
        if (best > ctx->guard_limit) {
            for (int v = u + 1; v < ctx->L; ++v) {
                if (!ctx->code[v].set) return NGC_ERR_STATE;
                double av[NGC_MAX_N] = {0.0};
                double rv = 0.0;
                ngc_layer_decode_vec(ctx, v, rows, ns, av, &rv);
                if (!(rv <= 1e-6)) continue;  // this layer cannot decode the set numerically: not a candidate
                const double kv = kappa_hat(v, av);
                if (kv < best) {
                    best = kv;
                    *layer_out = v;
                    for (int i = 0; i < n; ++i) a_out[i] = av[i];
                    if (residual_out) *residual_out = rv;
                }
                if (kv <= ctx->guard_limit) break;
            }
        }
    }
    return NGC_OK;
}

static int select_impl(const ngc_ctx* ctx, const uint8_t* mask, int* layer_out, double* a_out,
                       double* residual_out, bool first_only) {
    if (!ctx) return NGC_ERR_INVALID;
    if (!mask || !layer_out || !a_out) return ngc_fail(ctx, NGC_ERR_INVALID, "null argument");
    const int rc = ngc_select_core(ctx, mask, layer_out, a_out, residual_out, first_only);
    switch (rc) {
        case NGC_OK: return NGC_OK;
        case NGC_ERR_UNDECODABLE: return ngc_fail(ctx, rc, "stragglers exceed the largest tolerance");
        case NGC_ERR_STATE: return ngc_fail(ctx, rc, "chosen layer has no code yet");
        default: return ngc_fail(ctx, rc, "decode residual above tolerance");
    }
}

extern "C" int ngc_set_decode_guard(ngc_ctx* ctx, double kappa_limit) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!(kappa_limit >= 0.0)) return ngc_fail(ctx, NGC_ERR_INVALID, "the limit must be positive, or 0 to switch the guard off");
    ctx->guard_limit = std::isfinite(kappa_limit) ? kappa_limit : 0.0;  // no limit: the plain rule
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_select_decode_vec(const ngc_ctx* ctx, const uint8_t* straggler_mask, int* layer_out,
                                     double* a_out, double* residual_out) try {
    return select_impl(ctx, straggler_mask, layer_out, a_out, residual_out, false);
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_select_decode_vec_first(const ngc_ctx* ctx, const uint8_t* straggler_mask,
                                           int* layer_out, double* a_out, double* residual_out) try {
    return select_impl(ctx, straggler_mask, layer_out, a_out, residual_out, true);
} catch (...) {
    return ngc_on_exception();
}

// ---------------------------------------------------------------------------
// Redundancy-faithful execution (Sec. III, layered task scheduling; Sec. IV,
// termination): every worker works through its own partitions layer by layer.
// ---------------------------------------------------------------------------
int ngc_make_worker_plan(const ngc_ctx* ctx, ngc_worker_plan& plan) {
    const int n = ctx->n, L = ctx->L;
    for (int u = 0; u < L; ++u)
        if (!ctx->code[u].set) return ngc_fail(ctx, NGC_ERR_STATE, "a layer has no code yet");
    const int k = ctx->k, c = ctx->c;
    plan.order.assign(n, {});
    plan.needed.assign((size_t)L * n, 0);
    plan.T = 0;
    for (int i = 0; i < n; ++i) {
        std::vector<char> have(k, 0);
        for (int u = 0; u < L; ++u) {
            const std::vector<double>& B = ctx->code[u].B;
            int weight = 0;
            // a layer adds its new partitions in cyclic order starting at the worker's own group
            for (int t = 0; t < k; ++t) {
                const int j = (i * c + t) % k;
                if (B[(size_t)i * k + j] == 0.0) continue;
                ++weight;
                if (!have[j]) {
                    have[j] = 1;
                    plan.order[i].push_back(j);
                }
            }
            if (weight % c) return ngc_fail(ctx, NGC_ERR_INVALID, "a row's support is not a whole number of atomic tasks");
            plan.needed[(size_t)u * n + i] = weight / c;
        }
        plan.T = std::max(plan.T, (int)plan.order[i].size() / c);
    }
    return NGC_OK;
}

extern "C" int ngc_worker_task_count(const ngc_ctx* ctx, int* tasks_out) try {
    if (!ctx || !tasks_out) return NGC_ERR_INVALID;
    ngc_worker_plan plan;
    int rc = ngc_make_worker_plan(ctx, plan);
    if (rc) return rc;
    *tasks_out = plan.T;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_worker_schedule(const ngc_ctx* ctx, int worker, int* parts_out, int* count_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (worker < 0 || worker >= ctx->n || !parts_out || !count_out) return ngc_fail(ctx, NGC_ERR_INVALID, "bad worker or null output");
    ngc_worker_plan plan;
    int rc = ngc_make_worker_plan(ctx, plan);
    if (rc) return rc;
    *count_out = (int)plan.order[worker].size();
    for (size_t t = 0; t < plan.order[worker].size(); ++t) parts_out[t] = plan.order[worker][t];
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_select_from_progress(const ngc_ctx* ctx, const int* progress, int min_layer,
                                        int* layer_out, uint8_t* mask_out, double* a_out,
                                        double* residual_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!progress || !layer_out || !mask_out || !a_out) return ngc_fail(ctx, NGC_ERR_INVALID, "null argument");
    if (min_layer < 0 || min_layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "min_layer out of range");
    const int n = ctx->n;
    ngc_worker_plan plan;
    int rc = ngc_make_worker_plan(ctx, plan);
    if (rc) return rc;
    for (int i = 0; i < n; ++i) {
        a_out[i] = 0.0;
        mask_out[i] = 1;
        if (progress[i] < 0) return ngc_fail(ctx, NGC_ERR_INVALID, "negative progress");
    }
    *layer_out = -1;
    if (residual_out) *residual_out = 0.0;
    for (int u = min_layer; u < ctx->L; ++u) {
        int rows[NGC_MAX_N];
        int ns = 0;
        for (int i = 0; i < n; ++i)
            if (progress[i] >= plan.needed[(size_t)u * n + i]) rows[ns++] = i;
        if (ns < n - ctx->s[u]) continue;  // not enough finished workers for this component code
        *layer_out = u;
        for (int t = 0; t < ns; ++t) mask_out[rows[t]] = 0;
        double resid = 0.0;
        ngc_layer_decode_vec(ctx, u, rows, ns, a_out, &resid);
        if (residual_out) *residual_out = resid;
        if (!(resid <= 1e-6)) return ngc_fail(ctx, NGC_ERR_SINGULAR, "decode residual above tolerance");
        return NGC_OK;
    }
    return ngc_fail(ctx, NGC_ERR_UNDECODABLE, "no component code has enough finished workers");
} catch (...) {
    return ngc_on_exception();
}

// ---------------------------------------------------------------------------
// Explicit decoding matrix A_sigma (Def. 1): one row per straggler set of size
// sigma, supported on the n - sigma responders, with A_sigma B_sigma = 1.
// Rows are in lexicographic order of the (sorted) straggler sets.
// ---------------------------------------------------------------------------
static uint64_t binom_u64(int a, int b) {
    if (b < 0 || b > a) return 0;
    if (b > a - b) b = a - b;
    uint64_t r = 1;
    for (int i = 1; i <= b; ++i) {
        // r * (a - b + i) / i stays integral; guard against overflow
        const uint64_t f = (uint64_t)(a - b + i);
        if (r > UINT64_MAX / f) return UINT64_MAX;
        r = r * f / i;
    }
    return r;
}

// rank of the sorted subset c[0..sigma) of {0..n-1} among all subsets of that size
static int64_t subset_rank(const int* c, int sigma, int n) {
    uint64_t rank = 0;
    int prev = -1;
    for (int j = 0; j < sigma; ++j) {
        for (int v = prev + 1; v < c[j]; ++v) rank += binom_u64(n - 1 - v, sigma - 1 - j);
        prev = c[j];
    }
    return (int64_t)rank;
}

extern "C" int ngc_build_decoding_table(ngc_ctx* ctx, int layer, int64_t* rows_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "layer out of range");
    ngc_layer_code& lc = ctx->code[layer];
    if (!lc.set) return ngc_fail(ctx, NGC_ERR_STATE, "layer has no code yet");
    const int n = ctx->n, sigma = ctx->s[layer];
    const uint64_t rows = binom_u64(n, sigma);
    if (rows > (1ull << 20)) return ngc_fail(ctx, NGC_ERR_INVALID, "decoding table would exceed 2^20 rows");
    lc.A.assign((size_t)rows * n, 0.0);
    std::vector<int> out(sigma), resp(n);
    for (int j = 0; j < sigma; ++j) out[j] = j;
    for (uint64_t r = 0; r < rows; ++r) {
        int ns = 0, q = 0;
        for (int i = 0; i < n; ++i) {
            if (q < sigma && out[q] == i) { ++q; continue; }
            resp[ns++] = i;
        }
        double resid = 0.0;
        ngc_min_norm_decode(lc.B.data(), n, ctx->k, resp.data(), ns, &lc.A[(size_t)r * n], &resid);
        if (!(resid <= 1e-6)) {
            lc.A.clear();
            return ngc_fail(ctx, NGC_ERR_SINGULAR, "a straggler set of size sigma cannot be decoded");
        }
        // next subset in lexicographic order
        int j = sigma - 1;
        while (j >= 0 && out[j] == n - sigma + j) --j;
        if (j >= 0) {
            ++out[j];
            for (int t = j + 1; t < sigma; ++t) out[t] = out[t - 1] + 1;
        }
    }
    lc.A_rows = (int64_t)rows;
    lc.A_stale = true;
    if (rows_out) *rows_out = lc.A_rows;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_decoding_row_index(const ngc_ctx* ctx, int layer, const uint8_t* straggler_mask,
                                      int64_t* row_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->L || !straggler_mask || !row_out) return ngc_fail(ctx, NGC_ERR_INVALID, "bad layer or null argument");
    const int n = ctx->n, sigma = ctx->s[layer];
    int out[NGC_MAX_N];
    int cnt = 0;
    for (int i = 0; i < n; ++i)
        if (straggler_mask[i]) {
            if (cnt == sigma) return ngc_fail(ctx, NGC_ERR_UNDECODABLE, "more stragglers than this layer tolerates");
            out[cnt++] = i;
        }
    // fewer stragglers than sigma: the responders of highest index are left unused
    uint8_t used[NGC_MAX_N];
    for (int i = 0; i < n; ++i) used[i] = straggler_mask[i] != 0;
    for (int i = n - 1; i >= 0 && cnt < sigma; --i)
        if (!used[i]) { used[i] = 1; ++cnt; }
    cnt = 0;
    for (int i = 0; i < n; ++i)
        if (used[i]) out[cnt++] = i;
    *row_out = subset_rank(out, sigma, n);
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_get_decoding_row(const ngc_ctx* ctx, int layer, int64_t row, double* a_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->L || !a_out) return ngc_fail(ctx, NGC_ERR_INVALID, "bad layer or null output");
    const ngc_layer_code& lc = ctx->code[layer];
    if (lc.A_rows == 0) return ngc_fail(ctx, NGC_ERR_STATE, "no decoding table for this layer");
    if (row < 0 || row >= lc.A_rows) return ngc_fail(ctx, NGC_ERR_INVALID, "row out of range");
    std::memcpy(a_out, &lc.A[(size_t)row * ctx->n], sizeof(double) * ctx->n);
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}
