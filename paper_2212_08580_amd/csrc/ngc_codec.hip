// Encode, decode and the fused passes of libngc for gfx950 (CDNA4, wave64).
//
//  * encode (Sec. II-C, X = B G): a block stages a column tile of G (all k rows) in LDS
//    and writes messages from it, four workers at a time, so that a tile row read from
//    LDS feeds four messages;
//  * decode (Def. 1, A B = 1): the responders' messages are read once, products and sums
//    in fp64;
//  * coded rounds: encode of the chosen layer and decode of many rounds in one launch,
//    G read once per block, every message rounded to fp32, written, and combined from
//    registers;
//  * the tail of a whole iteration (block partials -> G -> messages -> decode -> update).
//
// All of them follow the canonical order of additions stated in ngc_dev_common.h, so the
// same inputs give the same bits whichever route computes them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <atomic>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

#include "ngc_dev_common.h"

// ---------------------------------------------------------------------------
// Code tables on the device.  Layout of d_code:
//   int   rowptr[L*n + 1] | int col[nnz] | float coef[nnz]      compressed rows, all layers
//   u32   gmask[L*ng]                (64-byte aligned)  bit t: one of the columns 4t..4t+3 is in the
//                                                       support of one of the workers 4g..4g+3
//   float gcoef[L*ng][kp/4][4][4]    (64-byte aligned)  gcoef[u*ng+g][j/4][r][j%4] = B^(u)[4g+r][j]: per trip
//                                                       of four columns, worker r's four coefficients together
// ng = ceil(n/4) groups of four workers, kp = k rounded up to a multiple of 4; rows and
// columns that do not exist hold zeros.
// ---------------------------------------------------------------------------
struct code_view {
    const int* rowptr;
    const int* col;
    const float* coef;
    const unsigned* gmask;
    const float* gcoef;
    int nnz, ng, kp;
};

static size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

static int upload_code(ngc_ctx* ctx) {
    if (!ctx->code_dirty && ctx->d_code) return NGC_OK;
    const int n = ctx->n, k = ctx->k, L = ctx->L;
    for (int u = 0; u < L; ++u)
        if (!ctx->code[u].set) return ngc_fail(ctx, NGC_ERR_STATE, "a layer has no code yet");
    size_t nnz = 0;
    for (int u = 0; u < L; ++u) nnz += ctx->code[u].col.size();
    const size_t np = (size_t)L * n;
    const int ng = (n + 3) / 4, kp = (k + 3) / 4 * 4;
    const size_t gmask_off = round_up((np + 1 + 2 * nnz) * sizeof(int), 64);
    const size_t gcoef_off = round_up(gmask_off + (size_t)L * ng * sizeof(unsigned), 64);
    const size_t bytes = gcoef_off + (size_t)L * ng * kp * 4 * sizeof(float);
    std::vector<unsigned char> host(bytes, 0);
    int* rowptr = reinterpret_cast<int*>(host.data());
    int* col = rowptr + np + 1;
    float* coef = reinterpret_cast<float*>(col + nnz);
    unsigned* gmask = reinterpret_cast<unsigned*>(host.data() + gmask_off);
    float* gcoef = reinterpret_cast<float*>(host.data() + gcoef_off);
    size_t at = 0;
    for (int u = 0; u < L; ++u) {
        const ngc_layer_code& lc = ctx->code[u];
        for (int i = 0; i < n; ++i) {
            rowptr[(size_t)u * n + i] = (int)at;
            const int g = i / 4, r = i % 4;
            for (int t = lc.rowptr[i]; t < lc.rowptr[i + 1]; ++t) {
                col[at] = lc.col[t];
                coef[at] = (float)lc.coef[t];
                gmask[(size_t)u * ng + g] |= 1u << (lc.col[t] / 4);
                gcoef[((size_t)u * ng + g) * kp * 4 + (size_t)(lc.col[t] / 4) * 16 + r * 4 + lc.col[t] % 4] = (float)lc.coef[t];
                ++at;
            }
        }
    }
    rowptr[np] = (int)at;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (bytes > ctx->d_code_bytes) {
        if (ctx->d_code) NGC_HIP(ctx, hipFree(ctx->d_code));
        ctx->d_code = nullptr;
        ctx->d_code_bytes = 0;
        if (hipMalloc(&ctx->d_code, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return ngc_fail(ctx, NGC_ERR_NOMEM, "code table allocation failed");
        }
        ctx->d_code_bytes = bytes;
    }
    NGC_HIP(ctx, hipMemcpy(ctx->d_code, host.data(), bytes, hipMemcpyHostToDevice));
    ctx->code_nnz = nnz;
    ctx->code_gmask_off = gmask_off;
    ctx->code_gcoef_off = gcoef_off;
    ctx->code_ng = ng;
    ctx->code_kp = kp;
    ctx->code_dirty = false;
    return NGC_OK;
}

static code_view view_code(const ngc_ctx* ctx) {
    code_view v;
    const size_t np = (size_t)ctx->L * ctx->n;
    const unsigned char* base = (const unsigned char*)ctx->d_code;
    v.rowptr = (const int*)base;
    v.col = v.rowptr + np + 1;
    v.coef = (const float*)(v.col + ctx->code_nnz);
    v.gmask = (const unsigned*)(base + ctx->code_gmask_off);
    v.gcoef = (const float*)(base + ctx->code_gcoef_off);
    v.nnz = (int)ctx->code_nnz;
    v.ng = ctx->code_ng;
    v.kp = ctx->code_kp;
    return v;
}

#include "ngc_codec_kernels.h"

// ===========================================================================
// host-side launchers
// ===========================================================================
extern "C" int ngc_encode(ngc_ctx* ctx, const float* G_dev, int layer, float* C_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!G_dev || !C_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null device pointer");
    if (layer < -1 || layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "layer out of range");
    if ((reinterpret_cast<uintptr_t>(G_dev) | reinterpret_cast<uintptr_t>(C_dev)) & 3)
        return ngc_fail(ctx, NGC_ERR_INVALID, "G and C must be 4-byte aligned");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    rc = upload_code(ctx);
    if (rc) return rc;
    const code_view cv = view_code(ctx);
    const int n = ctx->n;
    const int64_t d = ctx->d;
    const int lb = layer < 0 ? 0 : layer;
    const int lc = layer < 0 ? ctx->L : 1;
    const int V = ngc_vec_width(d, G_dev, C_dev);
    const int64_t gx = (d + 64 * V - 1) / (64 * V);
    const int items = lc * cv.ng;
    // about two blocks per CU; the (layer, group) items are dealt to blocks and waves in turn
    int64_t gy = std::max<int64_t>(1, (2 * (int64_t)ctx->cu_count + gx - 1) / gx);
    gy = std::min<int64_t>(gy, (items + ENC_WAVES - 1) / ENC_WAVES);
    if (gx > 0x7fffffffLL) return ngc_fail(ctx, NGC_ERR_INVALID, "d too large");
    dim3 grid((unsigned)gx, (unsigned)gy);
    const size_t lds = (size_t)cv.kp * 64 * V * sizeof(float);
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_ENCODE);
        if (V == 4)
            hipLaunchKernelGGL((encode_kernel<v4f, 4>), grid, dim3(ENC_WAVES * 64), lds, ctx->stream, G_dev, C_dev,
                               cv.gmask, cv.gcoef, n, ctx->k, cv.kp, cv.ng, d, lb, lc);
        else if (V == 2)
            hipLaunchKernelGGL((encode_kernel<v2f, 2>), grid, dim3(ENC_WAVES * 64), lds, ctx->stream, G_dev, C_dev,
                               cv.gmask, cv.gcoef, n, ctx->k, cv.kp, cv.ng, d, lb, lc);
        else
            hipLaunchKernelGGL((encode_kernel<float, 1>), grid, dim3(ENC_WAVES * 64), lds, ctx->stream, G_dev, C_dev,
                               cv.gmask, cv.gcoef, n, ctx->k, cv.kp, cv.ng, d, lb, lc);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// dense decode vector for the kernels; false if an entry is not finite
static bool fill_decode_args(const ngc_ctx* ctx, const double* a_host, decode_args& args, int* responders) {
    int cnt = 0;
    for (int i = 0; i < NGC_MAX_N; ++i) {
        const double a = i < ctx->n ? a_host[i] : 0.0;
        if (!std::isfinite(a)) return false;
        args.a[i] = a;
        cnt += a != 0.0;
    }
    if (responders) *responders = cnt;
    return true;
}

extern "C" int ngc_decode(ngc_ctx* ctx, int layer, const double* a_host, const float* C_dev,
                          float* g_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!a_host || !C_dev || !g_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (layer < 0 || layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "layer out of range");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    const int n = ctx->n;
    const int64_t d = ctx->d;
    decode_args args;
    int count = 0;
    if (!fill_decode_args(ctx, a_host, args, &count))
        return ngc_fail(ctx, NGC_ERR_INVALID, "decode vector has a non-finite entry");
    const float* Cl = C_dev + (size_t)layer * n * d;
    const int V = ngc_vec_width(d, Cl, g_dev);
    const int64_t gx = (d + 16 * V - 1) / (16 * V);
    const int64_t gw = (d + 256 * V - 1) / (256 * V);
    ngc_prof_scope ps(ctx, NGC_KERNEL_DECODE);
    if (count > 0 && gw >= 2 * (int64_t)ctx->cu_count) {
        // long gradient: enough column blocks to fill the chip with one thread per V columns
        if (V == 4)
            hipLaunchKernelGGL((decode_wide_kernel<v4f, 4>), dim3((unsigned)gw), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, args);
        else if (V == 2)
            hipLaunchKernelGGL((decode_wide_kernel<v2f, 2>), dim3((unsigned)gw), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, args);
        else
            hipLaunchKernelGGL((decode_wide_kernel<float, 1>), dim3((unsigned)gw), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, args);
    } else {
        if (V == 4)
            hipLaunchKernelGGL((decode_kernel<v4f, 4>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, args);
        else if (V == 2)
            hipLaunchKernelGGL((decode_kernel<v2f, 2>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, args);
        else
            hipLaunchKernelGGL((decode_kernel<float, 1>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, args);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---- coded rounds ---------------------------------------------------------------------------
// launch shape shared by the one-round and the many-round call
template <int MODE>
static int launch_rounds(ngc_ctx* ctx, const float* G_dev, int64_t g_stride, float* M_dev, int64_t m_stride,
                         float* g_dev, const round_rec* recs_dev, const round_rec& one, int rounds) {
    const code_view cv = view_code(ctx);
    const int64_t d = ctx->d;
    int V = ngc_vec_width(d, G_dev, M_dev);
    V = std::min(V, ngc_vec_width(d, g_dev, g_dev));
    if (g_stride % 4 || m_stride % 4) V = std::min(V, (g_stride % 2 || m_stride % 2) ? 1 : 2);
    // a single round has only its column tiles to fill the chip with: narrower tiles then
    if (MODE == ROUNDS_SINGLE)
        while (V > 1 && (d + 64 * V - 1) / (64 * V) < ctx->cu_count) V /= 2;
    const int64_t ntiles = (d + 64 * V - 1) / (64 * V);
    // runs of rounds per block: about four blocks per CU in all, two rounds of resident blocks (eight: 2 % slower,
    // a block then stages its tile for half as many rounds)
    int64_t chunks = std::max<int64_t>(1, std::min<int64_t>(rounds, (4 * (int64_t)ctx->cu_count + ntiles - 1) / ntiles));
    const int rpb = (int)((rounds + chunks - 1) / chunks);
    chunks = (rounds + rpb - 1) / rpb;
    if (ntiles * chunks > 0x7fffffffLL) return ngc_fail(ctx, NGC_ERR_INVALID, "too many column tiles times rounds");
    const size_t lds = (size_t)2 * 4 * 64 * V * sizeof(double) + (size_t)cv.kp * 64 * V * sizeof(float);
    if (lds > (size_t)ctx->lds_limit) return ngc_fail(ctx, NGC_ERR_INVALID, "tile does not fit the LDS of a block");
    dim3 grid((unsigned)(ntiles * chunks));
    ngc_prof_scope ps(ctx, NGC_KERNEL_ROUNDS);
#define NGC_ROUNDS_ARGS G_dev, g_stride, M_dev, m_stride, g_dev, recs_dev, one, cv.gmask, cv.gcoef, ctx->n, ctx->k, cv.kp, cv.ng, d, (int)ntiles, rounds, rpb
    if (V == 4)
        hipLaunchKernelGGL((coded_rounds_kernel<v4f, 4, MODE>), grid, dim3(256), lds, ctx->stream, NGC_ROUNDS_ARGS);
    else if (V == 2)
        hipLaunchKernelGGL((coded_rounds_kernel<v2f, 2, MODE>), grid, dim3(256), lds, ctx->stream, NGC_ROUNDS_ARGS);
    else
        hipLaunchKernelGGL((coded_rounds_kernel<float, 1, MODE>), grid, dim3(256), lds, ctx->stream, NGC_ROUNDS_ARGS);
#undef NGC_ROUNDS_ARGS
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
}

extern "C" int ngc_encode_decode(ngc_ctx* ctx, const float* G_dev, int layer, const double* a_host,
                                 float* M_dev, float* g_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!G_dev || !a_host || !M_dev || !g_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (layer < 0 || layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "layer out of range");
    if ((reinterpret_cast<uintptr_t>(G_dev) | reinterpret_cast<uintptr_t>(M_dev) | reinterpret_cast<uintptr_t>(g_dev)) & 3)
        return ngc_fail(ctx, NGC_ERR_INVALID, "device buffers must be 4-byte aligned");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    rc = upload_code(ctx);
    if (rc) return rc;
    round_rec one;
    std::memset(&one, 0, sizeof(one));
    for (int i = 0; i < ctx->n; ++i) {
        if (!std::isfinite(a_host[i])) return ngc_fail(ctx, NGC_ERR_INVALID, "decode vector has a non-finite entry");
        one.a[i] = a_host[i];
    }
    one.layer = layer;
    return launch_rounds<ROUNDS_SINGLE>(ctx, G_dev, 0, M_dev, 0, g_dev, nullptr, one, 1);
} catch (...) {
    return ngc_on_exception();
}

// room for `count` round records in the device table and its pinned staging copy
static int ensure_rounds(ngc_ctx* ctx, size_t count) {
    if (!ctx->rounds_ev) NGC_HIP(ctx, hipEventCreateWithFlags(&ctx->rounds_ev, hipEventDisableTiming));
    if (!ctx->rounds_copy_stream) NGC_HIP(ctx, hipStreamCreateWithFlags(&ctx->rounds_copy_stream, hipStreamNonBlocking));
    if (count <= ctx->rounds_cap) return NGC_OK;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->rounds_copy_stream));
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->d_rounds) NGC_HIP(ctx, hipFree(ctx->d_rounds));
    if (ctx->h_rounds) NGC_HIP(ctx, hipHostFree(ctx->h_rounds));
    ctx->d_rounds = ctx->h_rounds = nullptr;
    ctx->rounds_cap = 0;
    ctx->rounds_ev_set = false;
    const size_t cap = std::max<size_t>(count, 256);
    void* dp = nullptr;
    void* hp = nullptr;
    if (hipMalloc(&dp, cap * sizeof(round_rec)) != hipSuccess || hipHostMalloc(&hp, cap * sizeof(round_rec)) != hipSuccess) {
        (void)hipGetLastError();
        if (dp) (void)hipFree(dp);
        return ngc_fail(ctx, NGC_ERR_NOMEM, "round table allocation failed");
    }
    ctx->d_rounds = dp;
    ctx->h_rounds = hp;
    ctx->rounds_cap = cap;
    return NGC_OK;
}

extern "C" int ngc_coded_rounds(ngc_ctx* ctx, const float* G_dev, int64_t g_round_stride, int rounds,
                                const uint8_t* masks_host, float* M_dev, int64_t m_round_stride,
                                float* g_dev, int* layers_out, double* a_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!G_dev || !masks_host || !M_dev || !g_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (rounds < 1) return ngc_fail(ctx, NGC_ERR_INVALID, "rounds must be positive");
    const int n = ctx->n;
    const int64_t d = ctx->d;
    if (g_round_stride != 0 && g_round_stride < (int64_t)ctx->k * d)
        return ngc_fail(ctx, NGC_ERR_INVALID, "G round stride must be 0 (one G for all rounds) or at least k*d");
    if (rounds > 1 && m_round_stride < (int64_t)n * d)
        return ngc_fail(ctx, NGC_ERR_INVALID, "message round stride must be at least n*d");
    if ((reinterpret_cast<uintptr_t>(G_dev) | reinterpret_cast<uintptr_t>(M_dev) | reinterpret_cast<uintptr_t>(g_dev)) & 3)
        return ngc_fail(ctx, NGC_ERR_INVALID, "device buffers must be 4-byte aligned");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    rc = upload_code(ctx);
    if (rc) return rc;
    rc = ensure_rounds(ctx, (size_t)rounds);
    if (rc) return rc;
    // the staging copy is free once the previous call's transfer has finished
    if (ctx->rounds_ev_set) NGC_HIP(ctx, hipEventSynchronize(ctx->rounds_ev));
    round_rec* recs = (round_rec*)ctx->h_rounds;
    // main-node bookkeeping of every round up front (Observation after Def. 2; Def. 1): layer and
    // least-norm decode vector per mask, shared out over a few host threads
    std::vector<int> status((size_t)rounds, NGC_OK);
    std::atomic<bool> failed(false);
    auto plan = [&](int lo, int hi) {
        for (int r = lo; r < hi; ++r) {
            round_rec& rec = recs[r];
            std::memset(&rec, 0, sizeof(rec));
            int layer = -1;
            const int st = ngc_select_core(ctx, masks_host + (size_t)r * n, &layer, rec.a, nullptr, false);
            if (st == NGC_ERR_UNDECODABLE) {
                layer = -1;
            } else if (st != NGC_OK) {
                status[r] = st;
                layer = -1;
            }
            if (layer < 0)
                for (int i = 0; i < n; ++i) rec.a[i] = 0.0;
            rec.layer = layer;
        }
    };
    // The rounds go to the device in runs: a first short one of 64, so that the device starts
    // early, then runs of 256; while the kernel of one run works, the host solves for the next.
    // A round's bookkeeping costs about 0.3 + n^2 / 1500 microseconds; a pool thread (kept by the context, asleep
    // between calls) is worth waking per 40 microseconds of such work over the whole call, so
    // small jobs stay on the calling thread.  Each thread takes its share of every run and
    // counts itself done per run; the calling thread takes a share too, waits for the others,
    // copies the run's records and launches.
    std::vector<int> bounds{0};
    if (rounds >= 256) bounds.push_back(64);
    while (bounds.back() < rounds) bounds.push_back(std::min(rounds, bounds.back() + 256));
    const int nruns = (int)bounds.size() - 1;
    const unsigned hw = std::max(1u, std::thread::hardware_concurrency());
    const double work_us = (double)rounds * (0.3 + ctx->n * ctx->n / 1500.0);
    const int nthreads = (int)std::min<double>(std::min(hw, 16u), std::max(1.0, work_us / 40.0));
    std::unique_ptr<std::atomic<int>[]> done(new std::atomic<int>[nruns]);
    for (int c = 0; c < nruns; ++c) done[c].store(0);
    auto share_of_run = [&](int c, int tid) {
        const int lo = bounds[c], hi = bounds[c + 1];
        const int per = (hi - lo + nthreads - 1) / nthreads;
        plan(std::min(hi, lo + tid * per), std::min(hi, lo + (tid + 1) * per));
        done[c].fetch_add(1, std::memory_order_release);
    };
    // the pool's threads are waited for on every way out: they work on this call's arrays
    struct pool_guard {
        ngc_host_pool* p = nullptr;
        ~pool_guard() {
            if (p) p->wait();
        }
    } guard;
    if (nthreads > 1) {
        if (!ctx->pool) ctx->pool.reset(new ngc_host_pool);
        ctx->pool->start(nthreads - 1, [&](int tid) {
            int c = 0;
            try {
                for (; c < nruns; ++c) share_of_run(c, tid);
            } catch (...) {
                // out of memory inside a solve: its rounds stay unplanned, the call fails; the
                // runs this thread has not counted itself done for are counted now
                failed.store(true);
                for (; c < nruns; ++c) done[c].fetch_add(1, std::memory_order_release);
            }
        });
        guard.p = ctx->pool.get();
    }
    // Records are copied on the library's own stream: it first waits for what the caller's
    // stream holds now (kernels of an earlier call may still read the table), then a run's copy
    // can overlap the kernel of the run before it; the kernel waits for its run's copy.
    while ((int)ctx->rounds_run_ev.size() < nruns + 1) {
        hipEvent_t e = nullptr;
        NGC_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        ctx->rounds_run_ev.push_back(e);
    }
    NGC_HIP(ctx, hipEventRecord(ctx->rounds_run_ev[nruns], ctx->stream));
    NGC_HIP(ctx, hipStreamWaitEvent(ctx->rounds_copy_stream, ctx->rounds_run_ev[nruns], 0));
    round_rec none;
    std::memset(&none, 0, sizeof(none));
    for (int c = 0; c < nruns; ++c) {
        const int lo = bounds[c], hi = bounds[c + 1];
        share_of_run(c, 0);
        while (done[c].load(std::memory_order_acquire) < nthreads) std::this_thread::yield();
        if (failed.load()) return ngc_fail(ctx, NGC_ERR_NOMEM, "out of host memory while planning the rounds");
        for (int r = lo; r < hi; ++r) {
            if (status[r] != NGC_OK)
                return ngc_fail(ctx, status[r], status[r] == NGC_ERR_STATE ? "a chosen layer has no code yet"
                                                                           : "decode residual above tolerance in round " + std::to_string(r));
            if (layers_out) layers_out[r] = recs[r].layer;
            if (a_out) std::memcpy(a_out + (size_t)r * n, recs[r].a, sizeof(double) * n);
        }
        round_rec* d_recs = (round_rec*)ctx->d_rounds + lo;
        NGC_HIP(ctx, hipMemcpyAsync(d_recs, recs + lo, sizeof(round_rec) * (size_t)(hi - lo), hipMemcpyHostToDevice, ctx->rounds_copy_stream));
        NGC_HIP(ctx, hipEventRecord(ctx->rounds_run_ev[c], ctx->rounds_copy_stream));
        NGC_HIP(ctx, hipEventRecord(ctx->rounds_ev, ctx->rounds_copy_stream));  // the staging copy is free after this
        ctx->rounds_ev_set = true;
        NGC_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->rounds_run_ev[c], 0));
        if (g_round_stride != 0)
            rc = launch_rounds<ROUNDS_G_PER_ROUND>(ctx, G_dev + (int64_t)lo * g_round_stride, g_round_stride,
                                                   M_dev + (int64_t)lo * m_round_stride, m_round_stride,
                                                   g_dev + (int64_t)lo * d, d_recs, none, hi - lo);
        else
            rc = launch_rounds<ROUNDS_ONE_G>(ctx, G_dev, 0, M_dev + (int64_t)lo * m_round_stride, m_round_stride,
                                             g_dev + (int64_t)lo * d, d_recs, none, hi - lo);
        if (rc) return rc;
    }
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---- fused tail of ngc_iteration --------------------------------------------------------------
// LDS bytes of iteration_tail_kernel for vector width V, with or without the code tables
static size_t tail_lds_bytes(int n, int k, int L, size_t nnz, int V, bool tables) {
    size_t b = (size_t)16 * (16 * V + 1) * sizeof(double) + ((size_t)k + n) * 16 * V * sizeof(float);
    if (tables) b += ((size_t)L * n + 1 + 2 * nnz) * sizeof(int);
    return b;
}

extern "C" int ngc_tail_lds_bytes(const ngc_ctx* ctx, int vec_width, int64_t* with_tables_out,
                                  int64_t* without_tables_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (vec_width != 1 && vec_width != 2 && vec_width != 4) return ngc_fail(ctx, NGC_ERR_INVALID, "vector width must be 1, 2 or 4");
    size_t nnz = 0;
    for (int u = 0; u < ctx->L; ++u) {
        if (!ctx->code[u].set) return ngc_fail(ctx, NGC_ERR_STATE, "a layer has no code yet");
        nnz += ctx->code[u].col.size();
    }
    if (with_tables_out) *with_tables_out = (int64_t)tail_lds_bytes(ctx->n, ctx->k, ctx->L, nnz, vec_width, true);
    if (without_tables_out) *without_tables_out = (int64_t)tail_lds_bytes(ctx->n, ctx->k, ctx->L, nnz, vec_width, false);
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

int ngc_launch_tail(ngc_ctx* ctx, const float* partial, int chunks, int layer, const double* a,
                    float* G_dev, float* C_dev, float* g_dev, float* theta_dev, double scale) {
    int rc = upload_code(ctx);
    if (rc) return rc;
    const code_view cv = view_code(ctx);
    const int n = ctx->n, k = ctx->k, L = ctx->L;
    const int64_t d = ctx->d;
    decode_args args;
    if (!fill_decode_args(ctx, a, args, nullptr)) return ngc_fail(ctx, NGC_ERR_INVALID, "decode vector has a non-finite entry");
    // widest vector that still leaves about a block per four CUs
    int V = d % 4 == 0 ? 4 : (d % 2 == 0 ? 2 : 1);
    while (V > 1 && (d + 16 * V - 1) / (16 * V) < ctx->cu_count / 4) V /= 2;
    // the code tables go to LDS when they fit beside the tiles, else they stay in global memory;
    // a narrower vector shrinks the tiles if even those are too large
    bool tables = tail_lds_bytes(n, k, L, cv.nnz, V, true) <= (size_t)ctx->lds_limit;
    while (!tables && V > 1 && tail_lds_bytes(n, k, L, cv.nnz, V, false) > (size_t)ctx->lds_limit) V /= 2;
    const size_t lds = tail_lds_bytes(n, k, L, cv.nnz, V, tables);
    if (lds > (size_t)ctx->lds_limit) return ngc_fail(ctx, NGC_ERR_INVALID, "tiles do not fit the LDS of a block");
    const int64_t gx = (d + 16 * V - 1) / (16 * V);
    // The launch is short and bound by its chain of dependent steps, not by bytes: as many groups of
    // sixteen lanes as there are (layer, worker) messages to form, up to 64, shorten the chain.
    const int groups = (std::min(64, std::max(16, L * n)) + 3) / 4 * 4;  // whole waves
    const int threads = 16 * groups;
    ngc_prof_scope ps(ctx, NGC_KERNEL_TAIL);
#define NGC_TAIL_ARGS partial, chunks, G_dev, C_dev, cv.rowptr, cv.col, cv.coef, cv.nnz, n, k, L, d, layer, args, g_dev, theta_dev, (float)scale
#define NGC_TAIL_LAUNCH(VT, VV)                                                                                          \
    do {                                                                                                                 \
        if (tables)                                                                                                      \
            hipLaunchKernelGGL((iteration_tail_kernel<VT, VV, true>), dim3((unsigned)gx), dim3(threads), lds, ctx->stream, NGC_TAIL_ARGS); \
        else                                                                                                             \
            hipLaunchKernelGGL((iteration_tail_kernel<VT, VV, false>), dim3((unsigned)gx), dim3(threads), lds, ctx->stream, NGC_TAIL_ARGS); \
    } while (0)
    if (V == 4)
        NGC_TAIL_LAUNCH(v4f, 4);
    else if (V == 2)
        NGC_TAIL_LAUNCH(v2f, 2);
    else
        NGC_TAIL_LAUNCH(float, 1);
#undef NGC_TAIL_LAUNCH
#undef NGC_TAIL_ARGS
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
}

// ---- redundancy-faithful worker execution: messages from the workers' own gradients -----------
extern "C" int ngc_worker_encode(ngc_ctx* ctx, const float* W_dev, const int* progress_host,
                                 float* C_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!W_dev || !C_dev || !progress_host) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    ngc_worker_plan plan;
    rc = ngc_make_worker_plan(ctx, plan);
    if (rc) return rc;
    const int n = ctx->n, L = ctx->L, T = plan.T * ctx->c;  // T: partitions per worker schedule
    const int64_t d = ctx->d;
    worker_progress prog;
    for (int i = 0; i < NGC_MAX_N; ++i) prog.done[i] = 0;
    for (int i = 0; i < n; ++i) {
        if (progress_host[i] < 0) return ngc_fail(ctx, NGC_ERR_INVALID, "negative progress");
        prog.done[i] = (unsigned char)std::min<int>(progress_host[i], 255);
    }
    // tables: int needed[L*n] (atomic tasks) | int sched_len[n] (partitions) | float wcoef[L*n*T];
    // they depend on the code only
    if (ctx->wtab_dirty || !ctx->d_wtab || ctx->wtab_T != T) {
        const size_t head = (size_t)L * n + n;
        std::vector<int> tab(head + (size_t)L * n * T, 0);
        float* wcoef = reinterpret_cast<float*>(tab.data() + head);
        for (int i = 0; i < n; ++i) tab[(size_t)L * n + i] = (int)plan.order[i].size();
        for (int u = 0; u < L; ++u)
            for (int i = 0; i < n; ++i) {
                tab[(size_t)u * n + i] = plan.needed[(size_t)u * n + i];
                for (size_t t = 0; t < plan.order[i].size(); ++t)
                    wcoef[((size_t)u * n + i) * T + t] =
                        (float)ctx->code[u].B[(size_t)i * ctx->k + plan.order[i][t]];
            }
        NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (tab.size() * sizeof(int) > ctx->d_wtab_bytes) {
            if (ctx->d_wtab) NGC_HIP(ctx, hipFree(ctx->d_wtab));
            ctx->d_wtab = nullptr;
            ctx->d_wtab_bytes = 0;
            void* p = nullptr;
            if (hipMalloc(&p, tab.size() * sizeof(int)) != hipSuccess) {
                (void)hipGetLastError();
                return ngc_fail(ctx, NGC_ERR_NOMEM, "table allocation failed");
            }
            ctx->d_wtab = (int*)p;
            ctx->d_wtab_bytes = tab.size() * sizeof(int);
        }
        NGC_HIP(ctx, hipMemcpy(ctx->d_wtab, tab.data(), tab.size() * sizeof(int), hipMemcpyHostToDevice));
        ctx->wtab_dirty = false;
        ctx->wtab_T = T;
    }
    const int* needed = ctx->d_wtab;
    const int* sched_len = needed + (size_t)L * n;
    const float* wc = reinterpret_cast<const float*>(sched_len + n);
    const int V = ngc_vec_width(d, W_dev, C_dev);
    constexpr int LMAX = 8;  // layers per block: one pass over the worker's rows feeds eight accumulators
    dim3 grid((unsigned)((d + 64 * V - 1) / (64 * V)), (unsigned)n, (unsigned)((L + LMAX - 1) / LMAX));
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_ENCODE);
        if (V == 4)
            hipLaunchKernelGGL((worker_encode_kernel<v4f, 4, LMAX>), grid, dim3(64), 0, ctx->stream, W_dev, C_dev, needed, sched_len, wc, n, L, T, ctx->c, d, prog);
        else if (V == 2)
            hipLaunchKernelGGL((worker_encode_kernel<v2f, 2, LMAX>), grid, dim3(64), 0, ctx->stream, W_dev, C_dev, needed, sched_len, wc, n, L, T, ctx->c, d, prog);
        else
            hipLaunchKernelGGL((worker_encode_kernel<float, 1, LMAX>), grid, dim3(64), 0, ctx->stream, W_dev, C_dev, needed, sched_len, wc, n, L, T, ctx->c, d, prog);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---- decode through the explicit decoding matrix ------------------------------------------------
extern "C" int ngc_decode_lookup(ngc_ctx* ctx, int layer, const uint8_t* straggler_mask,
                                 const float* C_dev, float* g_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!straggler_mask || !C_dev || !g_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (layer < 0 || layer >= ctx->L) return ngc_fail(ctx, NGC_ERR_INVALID, "layer out of range");
    ngc_layer_code& lc = ctx->code[layer];
    if (lc.A_rows == 0) return ngc_fail(ctx, NGC_ERR_STATE, "call ngc_build_decoding_table for this layer first");
    int64_t row = 0;
    int rc = ngc_decoding_row_index(ctx, layer, straggler_mask, &row);
    if (rc) return rc;
    rc = ngc_dev_init(ctx);
    if (rc) return rc;
    const int n = ctx->n;
    const int64_t d = ctx->d;
    if (lc.A_stale || !lc.d_A) {
        NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (lc.d_A) NGC_HIP(ctx, hipFree(lc.d_A));
        lc.d_A = nullptr;
        void* p = nullptr;
        if (hipMalloc(&p, lc.A.size() * sizeof(double)) != hipSuccess) {
            (void)hipGetLastError();
            return ngc_fail(ctx, NGC_ERR_NOMEM, "decoding table allocation failed");
        }
        lc.d_A = (double*)p;
        NGC_HIP(ctx, hipMemcpy(lc.d_A, lc.A.data(), lc.A.size() * sizeof(double), hipMemcpyHostToDevice));
        lc.A_stale = false;
    }
    const float* Cl = C_dev + (size_t)layer * n * d;
    const double* a_row = lc.d_A + (size_t)row * n;
    const int V = ngc_vec_width(d, Cl, g_dev);
    const int64_t gx = (d + 16 * V - 1) / (16 * V);
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_DECODE);
        if (V == 4)
            hipLaunchKernelGGL((decode_lookup_kernel<v4f, 4>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, a_row);
        else if (V == 2)
            hipLaunchKernelGGL((decode_lookup_kernel<v2f, 2>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, a_row);
        else
            hipLaunchKernelGGL((decode_lookup_kernel<float, 1>), dim3((unsigned)gx), dim3(256), 0, ctx->stream, Cl, g_dev, d, n, a_row);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}
