// Latency model of Secs. II-D and IV: Monte-Carlo simulation of eq. (2) on the device (the
// closed forms of Lemma 1 and Theorem 1 are host code in ngc_latency_host.cpp).
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
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/ngc.h"

int ngc_on_exception();  // ngc_host.cpp: status for an exception caught at the C boundary
// ngc_latency_host.cpp: true if the model parameters are outside their documented ranges
bool ngc_latency_bad_params(int n, int s, double lam, double rho, double eps, double gamma, double pe);

namespace {

// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter-based generator
__host__ __device__ inline void philox4x32(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                           uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Values of each group of G consecutive lanes (G = 8, 16, 32 or 64) sorted in descending order
// over the group's lanes: a bitonic network of log2(G) (log2(G) + 1) / 2 compare-exchange steps;
// the partner's value comes through the cross-lane shuffle (LDS crossbar, not the vector ALU).
// idx = lane % G.  +-inf are ordinary values here, NaN does not occur.
template <int G>
__device__ __forceinline__ double group_sort_desc(double v, int idx) {
#pragma unroll
    for (int k = 2; k <= G; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const double pv = __shfl_xor(v, j, 64);
            // blocks of k lanes alternate between descending and ascending, the last pass
            // (k = G) is descending everywhere; the lane with the lower index of a pair keeps
            // the larger value in a descending block
            const bool desc = k == G || (idx & k) == 0;
            const bool lower = (idx & j) == 0;
            const double hi = fmax(v, pv), lo = fmin(v, pv);
            v = (lower == desc) ? hi : lo;
        }
    }
    return v;
}

// -log((w + 0.5) / 2^32) for a 32-bit word w, to about 2e-16 absolute.
// x = w + 0.5 = m 2^e with m in [1, 2); the top seven mantissa bits pick c = 1 + (i + 1/2)/128,
// and with r = m / c - 1 (|r| <= 2^-8, one fused multiply-add on the tabulated 1/c)
//   log x = e ln 2 + log c + log1p(r),
// log1p by its series up to r^6 (the next term is below 2e-18).  tab[i] = (1/c, -log(1/c)): the
// second entry belongs to the rounded first one, so the rounding of 1/c cancels.  ln 2 is split
// so that its multiples by the small integer 32 - e carry no rounding error worth the name.
__device__ __forceinline__ double neg_log_word(uint32_t w, const double2* __restrict__ tab) {
    const double x = (double)w + 0.5;  // exact
    const long long bits = __builtin_bit_cast(long long, x);
    const int e = (int)(bits >> 52) - 1023;
    const double m = __builtin_bit_cast(double, (bits & 0x000FFFFFFFFFFFFFLL) | 0x3FF0000000000000LL);
    const double2 t = tab[(int)(bits >> 45) & 127];
    const double r = fma(m, t.x, -1.0);
    double p = fma(r, -1.0 / 6.0, 1.0 / 5.0);
    p = fma(r, p, -1.0 / 4.0);
    p = fma(r, p, 1.0 / 3.0);
    p = fma(r, p, -1.0 / 2.0);
    p = fma(r, p, 1.0);
    const double ee = (double)(32 - e);
    constexpr double LN2_HI = 0x1.62e42fefa38p-1, LN2_LO = 0x1.ef35793c7673p-45;  // hi: 42 bits
    double acc = fma(ee, LN2_HI, -t.y);
    acc = fma(ee, LN2_LO, acc);
    return fma(-r, p, acc);
}

// A group of G lanes per trial (G = the smallest of 8, 16, 32, 64 that holds the n workers,
// so a wave runs 64 / G trials at once), lane = worker.  Word 0 of a worker's random stream
// decides failure, word u its u-th task time rho - log(U)/lambda (counter = (trial, worker,
// block, 0), key = seed; U = (word + 0.5) / 2^32).  For u = 1..top the u-th largest
// completion time of u tasks over the workers (= time at which n-u+1 workers have
// finished u tasks) is lane u-1 of the group's times sorted in descending order.
template <int G>
__global__ __launch_bounds__(256) void latency_sim_kernel(double* __restrict__ L,
                                                          double* __restrict__ Tmin, int n, int top,
                                                          double inv_lam, double rho, double eps,
                                                          double gamma, double pe, uint32_t k0,
                                                          uint32_t k1, int64_t trials) {
    constexpr int PER = 64 / G;  // trials per wave
    // table of the logarithm: one copy per block, from the library logarithm
    __shared__ double2 logtab[128];
    if (threadIdx.x < 128) {
        const double inv_c = 1.0 / (1.0 + ((double)threadIdx.x + 0.5) / 128.0);
        logtab[threadIdx.x] = make_double2(inv_c, -log(inv_c));
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int worker = lane % G, sub = lane / G;
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const double base = gamma + eps;
    for (int64_t rw = wave0 * PER; rw < trials; rw += nwaves * PER) {  // wave-uniform trip count
        const int64_t r = rw + sub;
        const bool live = r < trials;  // groups past the end idle along
        uint32_t w[4];
        philox4x32((uint32_t)r, (uint32_t)worker, 0u, 0u, k0, k1, w);
        const bool failed = ((double)w[0] + 0.5) / 4294967296.0 < pe;
        double cs = 0.0, best = INFINITY;
        for (int u = 1; u <= top; ++u) {
            if ((u & 3) == 0) philox4x32((uint32_t)r, (uint32_t)worker, (uint32_t)(u >> 2), 0u, k0, k1, w);
            cs += fma(neg_log_word(w[u & 3], logtab), inv_lam, rho);
            double v = failed ? INFINITY : base + cs;
            if (worker >= n) v = -INFINITY;
            const double Lu = __shfl(group_sort_desc<G>(v, worker), sub * G + (u - 1), 64);
            if (worker == 0 && live) L[(int64_t)(u - 1) * trials + r] = Lu;
            best = fmin(best, Lu);
        }
        if (Tmin && worker == 0 && live) Tmin[r] = best;
    }
}

}  // namespace

extern "C" int ngc_latency_simulate(void* hip_stream, int n, int smax, double lam, double rho, double eps,
                                    double gamma, double pe, uint64_t seed, int64_t trials,
                                    double* L_dev, double* Tngc_dev) try {
    if (ngc_latency_bad_params(n, smax, lam, rho, eps, gamma, pe) || !L_dev || trials < 1 || trials > 0xFFFFFFFFLL)
        return NGC_ERR_INVALID;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NGC_ERR_HIP;
    const int G = n <= 8 ? 8 : (n <= 16 ? 16 : (n <= 32 ? 32 : 64));  // lanes per trial
    const int64_t want = (trials + 4 * (64 / G) - 1) / (4 * (64 / G));
    const int64_t cap = (int64_t)(prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256) * 16;
    const unsigned blocks = (unsigned)(want < cap ? want : cap);
#define NGC_LATENCY_LAUNCH(GG)                                                                             \
    hipLaunchKernelGGL(latency_sim_kernel<GG>, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, L_dev, \
                       Tngc_dev, n, smax + 1, 1.0 / lam, rho, eps, gamma, pe, (uint32_t)seed,              \
                       (uint32_t)(seed >> 32), trials)
    if (G == 8)
        NGC_LATENCY_LAUNCH(8);
    else if (G == 16)
        NGC_LATENCY_LAUNCH(16);
    else if (G == 32)
        NGC_LATENCY_LAUNCH(32);
    else
        NGC_LATENCY_LAUNCH(64);
#undef NGC_LATENCY_LAUNCH
    return hipGetLastError() == hipSuccess ? NGC_OK : NGC_ERR_HIP;
} catch (...) {
    return ngc_on_exception();
}
