// Shared by the device-side sources of libngc (ngc_device.hip, ngc_codec.hip): vector types,
// the status macro for HIP calls, per-launch event records, and the canonical arithmetic of
// the encode and decode steps, which every kernel that forms messages or combines them must
// follow so that all routes give the same bits:
//
//   message   m_i[c] = fma(B[i][j], G[j][c], m_i[c]) over the columns j of B in ascending
//             order, one fp32 accumulator starting at +0 (a term whose coefficient is zero
//             leaves the accumulator as it is for finite G, so a kernel may skip it or not);
//   decode    responder i adds into partial sum number i mod 16, in ascending i:
//             s = fma(a_i, (double)m_i[c], s) in fp64; the sixteen partial sums are added as
//             q_w = ((s_4w + s_4w+1) + s_4w+2) + s_4w+3 for w = 0..3, then
//             ((q_0 + q_1) + q_2) + q_3, rounded once to fp32.
#pragma once

#include <hip/hip_runtime.h>

#include <string>

#include "ngc_internal.h"

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

#define NGC_HIP(ctx, call)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return ngc_fail(ctx, NGC_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

// defined in ngc_device.hip
int ngc_dev_init(ngc_ctx* ctx);

static inline bool ngc_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// widest vector (floats) that the length and both pointers allow
static inline int ngc_vec_width(int64_t d, const void* p0, const void* p1) {
    auto al = [](const void* p, uintptr_t m) { return (reinterpret_cast<uintptr_t>(p) & (m - 1)) == 0; };
    if (d % 4 == 0 && al(p0, 16) && al(p1, 16)) return 4;
    if (d % 2 == 0 && al(p0, 8) && al(p1, 8)) return 2;
    return 1;
}

// Brackets the launches made during its lifetime with a pair of events on the context's
// stream when the kernel id is selected for timing.
struct ngc_prof_scope {
    ngc_ctx* ctx;
    int rec = -1;
    ngc_prof_scope(ngc_ctx* c, int kernel) : ctx(c) {
        if (c->prof_suspended || !((c->profile_mask >> kernel) & 1u) || c->prof.size() >= (size_t)NGC_MAX_PROFILE) return;
        ngc_profile_rec r;
        r.kernel = kernel;
        auto get = [&](hipEvent_t& e) {
            if (!c->event_pool.empty()) {
                e = c->event_pool.back();
                c->event_pool.pop_back();
                return true;
            }
            return hipEventCreate(&e) == hipSuccess;
        };
        if (!get(r.start)) return;
        if (!get(r.stop)) {
            c->event_pool.push_back(r.start);
            return;
        }
        (void)hipEventRecord(r.start, c->stream);
        c->prof.push_back(r);
        rec = (int)c->prof.size() - 1;
    }
    ~ngc_prof_scope() {
        if (rec >= 0) (void)hipEventRecord(ctx->prof[rec].stop, ctx->stream);
    }
    ngc_prof_scope(const ngc_prof_scope&) = delete;
    ngc_prof_scope& operator=(const ngc_prof_scope&) = delete;
};

// ---- element-wise helpers on 1, 2 or 4 floats -------------------------------------------
template <typename VT> struct ngc_vec;
template <> struct ngc_vec<float> { static constexpr int V = 1; };
template <> struct ngc_vec<v2f> { static constexpr int V = 2; };
template <> struct ngc_vec<v4f> { static constexpr int V = 4; };

__device__ __forceinline__ float ngc_get(float x, int) { return x; }
__device__ __forceinline__ float ngc_get(v2f x, int v) { return x[v]; }
__device__ __forceinline__ float ngc_get(v4f x, int v) { return x[v]; }
__device__ __forceinline__ void ngc_set(float& x, int, float s) { x = s; }
__device__ __forceinline__ void ngc_set(v2f& x, int v, float s) { x[v] = s; }
__device__ __forceinline__ void ngc_set(v4f& x, int v, float s) { x[v] = s; }

// m <- fma(w, x, m) component by component (an explicit fused multiply-add: the same
// instruction in every kernel, whatever the compiler's contraction setting)
__device__ __forceinline__ float ngc_fma(float w, float x, float m) { return __builtin_fmaf(w, x, m); }
__device__ __forceinline__ v2f ngc_fma(float w, v2f x, v2f m) {
    v2f r;
    r.x = __builtin_fmaf(w, x.x, m.x);
    r.y = __builtin_fmaf(w, x.y, m.y);
    return r;
}
__device__ __forceinline__ v4f ngc_fma(float w, v4f x, v4f m) {
    v4f r;
    r.x = __builtin_fmaf(w, x.x, m.x);
    r.y = __builtin_fmaf(w, x.y, m.y);
    r.z = __builtin_fmaf(w, x.z, m.z);
    r.w = __builtin_fmaf(w, x.w, m.w);
    return r;
}

// the canonical combination of sixteen fp64 partial sums s[0..15] (see the top of this file)
__device__ __forceinline__ double ngc_quad(double s0, double s1, double s2, double s3) {
    return ((s0 + s1) + s2) + s3;
}
