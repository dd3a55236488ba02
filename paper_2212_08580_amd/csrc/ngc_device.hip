// Device side of libngc for gfx950 (CDNA4, wave64): partition gradients and the
// descent update, their launchers, per-kernel timing and the measurement probes.
// Encode, decode and the fused passes are in ngc_codec.hip.
//
// Bandwidth picture (fp32 everywhere on the device): partition gradients read every
// row of X from HBM exactly once; all other traffic (theta, labels, block partials,
// G) is below 2 % of that.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>

#include "ngc_dev_common.h"

#include "ngc_grad_kernels.h"
#include "ngc_grad_flat.h"

// ===========================================================================
// host-side launchers
// ===========================================================================
int ngc_dev_init(ngc_ctx* ctx) {
    if (ctx->dev_ready) return NGC_OK;
    int dev = 0;
    NGC_HIP(ctx, hipGetDevice(&dev));
    hipDeviceProp_t prop;
    NGC_HIP(ctx, hipGetDeviceProperties(&prop, dev));
    ctx->cu_count = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    ctx->lds_limit = prop.sharedMemPerBlock > 0 ? (int)std::min<size_t>(prop.sharedMemPerBlock, 160 * 1024) : 64 * 1024;
    ctx->dev_ready = true;
    return NGC_OK;
}

void ngc_dev_release(ngc_ctx* ctx) {
    if (!ctx->dev_ready) return;
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& r : ctx->prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (auto e : ctx->event_pool) (void)hipEventDestroy(e);
    if (ctx->d_code) (void)hipFree(ctx->d_code);
    if (ctx->d_ws) (void)hipFree(ctx->d_ws);
    for (int q = 0; q < 2; ++q) {
        if (ctx->d_maps[q]) (void)hipFree(ctx->d_maps[q]);
        if (ctx->h_maps[q]) (void)hipHostFree(ctx->h_maps[q]);
        if (ctx->maps_ev[q]) (void)hipEventDestroy(ctx->maps_ev[q]);
        ctx->d_maps[q] = ctx->h_maps[q] = nullptr;
        ctx->maps_ev[q] = nullptr;
        ctx->maps_ev_set[q] = false;
    }
    ctx->maps_cap = 0;
    if (ctx->d_rounds) (void)hipFree(ctx->d_rounds);
    if (ctx->h_rounds) (void)hipHostFree(ctx->h_rounds);
    if (ctx->rounds_ev) (void)hipEventDestroy(ctx->rounds_ev);
    if (ctx->rounds_copy_stream) {
        (void)hipStreamSynchronize(ctx->rounds_copy_stream);
        (void)hipStreamDestroy(ctx->rounds_copy_stream);
    }
    ctx->rounds_copy_stream = nullptr;
    for (auto e : ctx->rounds_run_ev) (void)hipEventDestroy(e);
    ctx->rounds_run_ev.clear();
    ctx->d_rounds = ctx->h_rounds = nullptr;
    ctx->rounds_ev = nullptr;
    ctx->rounds_ev_set = false;
    ctx->rounds_cap = 0;
    if (ctx->d_wtab) (void)hipFree(ctx->d_wtab);
    ctx->d_wtab = nullptr;
    ctx->d_wtab_bytes = 0;
    ctx->wtab_dirty = true;
    for (auto& lc : ctx->code) {
        if (lc.d_A) (void)hipFree(lc.d_A);
        lc.d_A = nullptr;
        lc.A_stale = true;
    }
    ctx->d_code = nullptr;
    ctx->d_ws = nullptr;
    ctx->dev_ready = false;
}

static int ensure_ws(ngc_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->d_ws_bytes) return NGC_OK;
    if (ctx->d_ws) {
        NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
        NGC_HIP(ctx, hipFree(ctx->d_ws));
        ctx->d_ws = nullptr;
        ctx->d_ws_bytes = 0;
    }
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return ngc_fail(ctx, NGC_ERR_NOMEM, "workspace allocation failed");
    }
    ctx->d_ws = (float*)p;
    ctx->d_ws_bytes = bytes;
    return NGC_OK;
}

extern "C" int ngc_profile_enable(ngc_ctx* ctx, int kernel_mask) try {
    if (!ctx) return NGC_ERR_INVALID;
    ctx->profile_mask = (unsigned)kernel_mask;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_profile_read(ngc_ctx* ctx, int64_t* launches_out, double* total_ms_out) try {
    if (!ctx || !launches_out || !total_ms_out) return NGC_ERR_INVALID;
    for (int i = 0; i < NGC_KERNEL_COUNT; ++i) {
        launches_out[i] = 0;
        total_ms_out[i] = 0.0;
    }
    if (ctx->prof.empty()) return NGC_OK;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (auto& r : ctx->prof) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            launches_out[r.kernel] += 1;
            total_ms_out[r.kernel] += ms;
        }
        ctx->event_pool.push_back(r.start);
        ctx->event_pool.push_back(r.stop);
    }
    ctx->prof.clear();
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_profile_launches(ngc_ctx* ctx, int kernel, double* ms_out, int64_t capacity,
                                    int64_t* count_out) try {
    if (!ctx || !count_out || capacity < 0 || (capacity > 0 && !ms_out)) return NGC_ERR_INVALID;
    if (kernel < 0 || kernel >= NGC_KERNEL_COUNT) return ngc_fail(ctx, NGC_ERR_INVALID, "unknown kernel id");
    *count_out = 0;
    if (ctx->prof.empty()) return NGC_OK;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    int64_t seen = 0;
    for (auto& r : ctx->prof) {
        if (r.kernel != kernel) continue;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
        if (seen < capacity) ms_out[seen] = ms;
        ++seen;
    }
    *count_out = seen;
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_sync(ngc_ctx* ctx) try {
    if (!ctx) return NGC_ERR_INVALID;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}


// ---- partition gradients --------------------------------------------------
template <int NV, int R, int NBUF, int WAVES, bool RAGGED, typename VT = v4f, bool TH_LDS = false>
static void launch_stream(ngc_ctx* ctx, int loss, const float* X, const float* y,
                          const float* theta, float* partial, int k, int64_t rows, int chunks,
                          int64_t rpc, const int* unit_part, int dq) {
    dim3 grid((unsigned)(k * chunks));
    if (loss == NGC_LOSS_LSQ)
        hipLaunchKernelGGL((grad_stream_kernel<NV, R, NBUF, WAVES, NGC_LOSS_LSQ, RAGGED, VT, TH_LDS>), grid,
                           dim3(WAVES * 64), 0, ctx->stream, X, y, theta, partial, rows, chunks, rpc,
                           unit_part, dq);
    else
        hipLaunchKernelGGL((grad_stream_kernel<NV, R, NBUF, WAVES, NGC_LOSS_LOGISTIC, RAGGED, VT, TH_LDS>), grid,
                           dim3(WAVES * 64), 0, ctx->stream, X, y, theta, partial, rows, chunks, rpc,
                           unit_part, dq);
}

// Shape of the single-pass kernel for a given d, or waves = 0 if d has none
// (above 32768, or above 16384 and not a multiple of 4).  A block offers
// nv*waves*64 slots per row, each a float4, or a float (`scalar`) when d is not
// a multiple of 4 and rows are therefore not 16-byte aligned; `ragged` when
// the row has fewer elements than the block has slots.
struct stream_shape {
    int nv, r, waves;
    bool ragged, scalar;
    int narrow_dq = 0;  // > 0: rows of narrow_dq elements take a kernel that loads several rows at once
    bool narrow_any = false;  // narrow_dq counts single floats (scalar): grad_narrow_any_kernel
    int flat_dmax = 0;        // > 0: grad_flat_kernel<flat_dmax, flat_lanes> (rows read as one flat stretch of float4)
    int flat_lanes = 1;       // lanes that share a row
};
// allow_flat: X holds at least one whole float4
static stream_shape pick_stream_shape(int64_t d, bool allow_flat) {
    if (d % 4 == 0 && d <= 128 && ((d / 4) & (d / 4 - 1)) == 0) return {1, 8, 1, false, false, (int)(d / 4)};
    // every other row of fewer than 64 features, 16-byte addressable or not: read as one flat stretch,
    // 64 * (64 / dmax) whole rows per trip and wave (48 features with padded rows in LDS, or its
    // reads would collide sixteen-way)
    if (allow_flat && d < 64) {
        const int dmax = d < 2 ? 2 : 8 * (int)(d / 8 + 1);  // (4 for d = 3: 6.3 -> 5.8 TB/s)
        return {1, 1, 1, false, true, 0, false, dmax};
    }
    // the same, four or eight lanes to a row, for rows of 65 to 248 features that are no multiple
    // of 4 and for the multiples of 4 up to 132 (from 144 on the kernel with one float4 per lane
    // and row is as fast: 6.7-6.85 TB/s)
    if (allow_flat && d > 64 && d <= 248 && (d % 4 != 0 || d <= 132)) {
        const int lanes = d <= 124 ? 4 : 8;
        const int h = (int)((d + lanes - 1) / lanes);  // 16 .. 31
        return {1, 1, 1, false, true, 0, false, 8 * (h / 8 + 1), lanes};
    }
    // an X of fewer than four floats (at most three features): two or more whole rows per wave-wide load
    if (d % 4 != 0 && d <= 21) return {1, 8, 1, false, true, (int)d, true};
    if (d % 1024 == 0) {
        const int w = (int)(d / 1024);
        // narrow rows: one float4 per lane and many waves per block rather than one wave with
        // four; the kernel runs as fast and leaves a quarter of the block partials to be summed
        if (w == 1 || w == 2) return {1, 16, 4 * w, false, false};
        if (w == 3) return {3, 5, 4, false, false};  // four waves fill a CU's eight wave slots, three do not
        if (w == 4 || w == 6 || w == 8) return {4, 4, w, false, false};
        if (w == 12 || w == 16) return {8, 2, w / 2, false, false};
    }
    if (d == 256) return {1, 16, 1, false, false};
    if (d == 512) return {2, 8, 1, false, false};
    if (d == 768) return {3, 5, 1, false, false};
    // wide rows: ten to sixteen waves of eight float4 per lane and row, theta in LDS (the shapes with more than eight waves)
    if (d > 16384 && d <= 32768 && d % 4 == 0) return {8, 1, 2 * (int)((d / 4 + 1023) / 1024), true, false};
    if (d < 1 || d > 16384) return {0, 0, 0, false, false};
    if (d % 4 != 0) {
        if (d <= 256) return {4, 16, 1, true, true};  // 249 .. 255 (shorter rows are read as a flat stretch)
        if (d <= 4096) return {8, 8, (int)((d + 511) / 512), true, true};
        if (d <= 8192) return {16, 3, (int)((d + 1023) / 1024), true, true};
        // up to 16384: ten, twelve or sixteen waves, theta in LDS, one row per group (fourteen waves
        // spill a dozen registers and are slower than sixteen with idle slots: 5.2 against 5.5 TB/s)
        return {16, 1, d <= 10240 ? 10 : d <= 12288 ? 12 : 16, true, true};
    }
    const int dq = (int)(d / 4);
    if (dq <= 64) return {1, 16, 1, true, false};
    if (dq <= 128) return {2, 8, 1, true, false};
    if (dq <= 192) return {3, 5, 1, true, false};
    if (dq > 512 && dq <= 768) return {3, 5, 4, true, false};
    if (dq <= 2048) return {4, 4, (dq + 255) / 256, true, false};
    return {8, 2, (dq + 511) / 512, true, false};
}

int ngc_mlp2_grads(ngc_ctx* ctx, const float* X, const int* labels, const float* theta, int64_t rows,
                   float* G, int units, const int* unit_part, const int* unit_row);  // ngc_mlp.hip
// ngc_codec.hip: everything of an iteration after the gradient kernel, in one launch
int ngc_launch_tail(ngc_ctx* ctx, const float* partial, int chunks, int layer, const double* a,
                    float* G_dev, float* C_dev, float* g_dev, float* theta_dev, double scale);

// Gradients of `units` partial-gradient computations (least squares / logistic).  Unit q works
// on partition unit_part[q] (q itself if unit_part is null) and its result goes to row
// unit_row[q] of G_dev (row q if null); both maps are device arrays.
struct partial_info {
    const float* ptr = nullptr;  // [units][chunks][d]
    int chunks = 0;
};

// If `defer` is given the block partials are left unreduced for the caller to sum (in chunk
// order) and G_dev is not written.
// With `fixed_ws` the block partials go to that buffer of fixed_bytes bytes instead of the
// context's workspace, nothing is allocated, and a need beyond it is NGC_ERR_INVALID.
static int grads_impl(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                      const float* theta_dev, int64_t rows, float* G_dev, int units,
                      const int* unit_part, const int* unit_row, partial_info* defer = nullptr,
                      float* fixed_ws = nullptr, size_t fixed_bytes = 0) {
    int rc = NGC_OK;
    float* ws = nullptr;
    auto get_ws = [&](size_t bytes) -> int {
        if (fixed_ws) {
            if (bytes > fixed_bytes)
                return ngc_fail(ctx, NGC_ERR_INVALID,
                                "this shape needs " + std::to_string(bytes) + " bytes of scratch, the static scratch holds " +
                                    std::to_string(fixed_bytes));
            ws = fixed_ws;
            return NGC_OK;
        }
        const int e = ensure_ws(ctx, bytes);
        ws = ctx->d_ws;
        return e;
    };
    const int k = units;
    const int64_t d = ctx->d;
    const float* y = (const float*)y_dev;
    const int64_t wave_slots = (int64_t)ctx->cu_count * 8;  // 2 waves per SIMD

    const int64_t x_floats = (int64_t)ctx->k * rows * d;
    const stream_shape sh = pick_stream_shape(d, x_floats >= 4);
    if (sh.waves) {
        // enough blocks to give every SIMD two waves, split evenly over the partitions
        // a CU holds 8 such waves (2 per SIMD at up to 256 registers), so it takes
        // 8 / waves whole blocks; more blocks than that would run as a second,
        // partly filled round
        // rows of at most 128 features fill no more than half of a wave's lanes: twice the
        // blocks keep as many bytes in flight (measured: 3.1 -> 3.6 TB/s at 64 features,
        // 4.3 -> 5.0 at 100, 5.5 -> 6.1 at 128; wider rows lose 2 % with more than 8)
        // (the flat kernel's blocks are four waves with 16 KiB of LDS each: two per CU)
        const int per_cu = sh.flat_dmax ? 2 : (sh.waves == 1 && d <= 128) ? 16 : std::max(1, 8 / sh.waves);
        const int64_t block_slots = (int64_t)ctx->cu_count * per_cu;
        int64_t chunks = std::max<int64_t>(1, block_slots / k);
        int64_t rpc = (rows + chunks - 1) / chunks;
        // two row groups: one trip of the kernel's loop (a narrow-row group is r loads of 64/dq rows)
        const int64_t quantum = sh.flat_dmax ? 4 * (64 / sh.flat_lanes) * (64 / sh.flat_dmax) : sh.narrow_dq ? 2 * sh.r * (64 / sh.narrow_dq) : 2 * sh.r;
        rpc = ((rpc + quantum - 1) / quantum) * quantum;
        chunks = (rows + rpc - 1) / rpc;
        rc = get_ws(sizeof(float) * (size_t)k * chunks * d);
        if (rc) return rc;
        {
            ngc_prof_scope ps(ctx, NGC_KERNEL_GRAD);
#define NGC_STREAM_ARGS ctx, loss, X_dev, y, theta_dev, ws, k, rows, (int)chunks, rpc, unit_part, (int)(sh.scalar ? d : d / 4)
#define NGC_STREAM_CASE(NV, R, W, RG) \
    case W: launch_stream<NV, R, 2, W, RG>(NGC_STREAM_ARGS); break;
#define NGC_STREAM_SCALAR(NV, R, W) \
    case W: launch_stream<NV, R, 2, W, true, float>(NGC_STREAM_ARGS); break;
            if (sh.flat_dmax) {
                dim3 grid((unsigned)(k * chunks));
#define NGC_FLAT_CASE(DMAX, LANES)                                                                                  \
    case DMAX * 16 + LANES:                                                                                         \
        if (loss == NGC_LOSS_LSQ)                                                                                   \
            hipLaunchKernelGGL((grad_flat_kernel<DMAX, LANES, NGC_LOSS_LSQ>), grid, dim3(256), 0, ctx->stream,      \
                               X_dev, y, theta_dev, ws, rows, (int)chunks, rpc, unit_part, (int)d, x_floats);       \
        else                                                                                                        \
            hipLaunchKernelGGL((grad_flat_kernel<DMAX, LANES, NGC_LOSS_LOGISTIC>), grid, dim3(256), 0, ctx->stream, \
                               X_dev, y, theta_dev, ws, rows, (int)chunks, rpc, unit_part, (int)d, x_floats);       \
        break;
#define NGC_FLAT_PAD_CASE(DMAX)                                                                                      \
    case DMAX:                                                                                                       \
        if (loss == NGC_LOSS_LSQ)                                                                                    \
            hipLaunchKernelGGL((grad_flat_kernel<DMAX, 1, NGC_LOSS_LSQ, true>), grid, dim3(256), 0, ctx->stream,     \
                               X_dev, y, theta_dev, ws, rows, (int)chunks, rpc, unit_part, (int)d, x_floats);        \
        else                                                                                                         \
            hipLaunchKernelGGL((grad_flat_kernel<DMAX, 1, NGC_LOSS_LOGISTIC, true>), grid, dim3(256), 0, ctx->stream, \
                               X_dev, y, theta_dev, ws, rows, (int)chunks, rpc, unit_part, (int)d, x_floats);        \
        break;
                if (d == 48) {  // padded rows in LDS (for 24, 40 and 56 features they change nothing measurable)
                    switch (sh.flat_dmax) { NGC_FLAT_PAD_CASE(56) }
                } else
                switch (sh.flat_dmax * 16 + sh.flat_lanes) {
                    NGC_FLAT_CASE(2, 1) NGC_FLAT_CASE(8, 1) NGC_FLAT_CASE(16, 1) NGC_FLAT_CASE(24, 1)
                    NGC_FLAT_CASE(32, 1) NGC_FLAT_CASE(40, 1) NGC_FLAT_CASE(48, 1) NGC_FLAT_CASE(56, 1)
                    NGC_FLAT_CASE(64, 1) NGC_FLAT_CASE(24, 4) NGC_FLAT_CASE(32, 4) NGC_FLAT_CASE(24, 8)
                    NGC_FLAT_CASE(32, 8)
                }
#undef NGC_FLAT_CASE
#undef NGC_FLAT_PAD_CASE
            } else if (sh.narrow_any) {
                dim3 grid((unsigned)(k * chunks));
#define NGC_NARROW_ANY(VT, RR, LOSS_ID)                                                                            \
    hipLaunchKernelGGL((grad_narrow_any_kernel<VT, RR, LOSS_ID>), grid, dim3(64), 0, ctx->stream, X_dev, y, theta_dev, \
                       ws, rows, (int)chunks, rpc, unit_part, sh.narrow_dq)
                if (loss == NGC_LOSS_LSQ) NGC_NARROW_ANY(float, 8, NGC_LOSS_LSQ); else NGC_NARROW_ANY(float, 8, NGC_LOSS_LOGISTIC);
#undef NGC_NARROW_ANY
            } else if (sh.narrow_dq) {
                dim3 grid((unsigned)(k * chunks));
#define NGC_NARROW_CASE(DQ)                                                                                          \
    case DQ:                                                                                                         \
        if (loss == NGC_LOSS_LSQ)                                                                                    \
            hipLaunchKernelGGL((grad_narrow_kernel<DQ, 8, NGC_LOSS_LSQ>), grid, dim3(64), 0, ctx->stream, X_dev, y,  \
                               theta_dev, ws, rows, (int)chunks, rpc, unit_part);                                    \
        else                                                                                                         \
            hipLaunchKernelGGL((grad_narrow_kernel<DQ, 8, NGC_LOSS_LOGISTIC>), grid, dim3(64), 0, ctx->stream, X_dev, \
                               y, theta_dev, ws, rows, (int)chunks, rpc, unit_part);                                 \
        break;
                switch (sh.narrow_dq) {
                    NGC_NARROW_CASE(1) NGC_NARROW_CASE(2) NGC_NARROW_CASE(4) NGC_NARROW_CASE(8)
                    NGC_NARROW_CASE(16) NGC_NARROW_CASE(32)
                }
#undef NGC_NARROW_CASE
            } else if (sh.scalar) {
                if (sh.nv == 4) {
                    launch_stream<4, 16, 2, 1, true, float>(NGC_STREAM_ARGS);
                } else if (sh.nv == 8) {
                    switch (sh.waves) {
                        NGC_STREAM_SCALAR(8, 8, 1) NGC_STREAM_SCALAR(8, 8, 2) NGC_STREAM_SCALAR(8, 8, 3)
                        NGC_STREAM_SCALAR(8, 8, 4) NGC_STREAM_SCALAR(8, 8, 5) NGC_STREAM_SCALAR(8, 8, 6)
                        NGC_STREAM_SCALAR(8, 8, 7) NGC_STREAM_SCALAR(8, 8, 8)
                    }
                } else {
                    switch (sh.waves) {
                        NGC_STREAM_SCALAR(16, 3, 5) NGC_STREAM_SCALAR(16, 3, 6)
                        NGC_STREAM_SCALAR(16, 3, 7) NGC_STREAM_SCALAR(16, 3, 8)
                        case 10: launch_stream<16, 1, 2, 10, true, float, true>(NGC_STREAM_ARGS); break;
                        case 12: launch_stream<16, 1, 2, 12, true, float, true>(NGC_STREAM_ARGS); break;
                        case 16: launch_stream<16, 1, 2, 16, true, float, true>(NGC_STREAM_ARGS); break;
                    }
                }
            } else if (!sh.ragged) {
                if (sh.nv == 4) {
                    switch (sh.waves) {
                        NGC_STREAM_CASE(4, 4, 4, false) NGC_STREAM_CASE(4, 4, 6, false)
                        NGC_STREAM_CASE(4, 4, 8, false)
                    }
                } else if (sh.nv == 8) {
                    switch (sh.waves) {
                        NGC_STREAM_CASE(8, 2, 6, false) NGC_STREAM_CASE(8, 2, 8, false)
                    }
                } else if (sh.nv == 1) {
                    switch (sh.waves) {
                        NGC_STREAM_CASE(1, 16, 1, false) NGC_STREAM_CASE(1, 16, 4, false)
                        NGC_STREAM_CASE(1, 16, 8, false)
                    }
                } else if (sh.nv == 2) {
                    launch_stream<2, 8, 2, 1, false>(NGC_STREAM_ARGS);
                } else if (sh.waves == 4) {
                    launch_stream<3, 5, 2, 4, false>(NGC_STREAM_ARGS);
                } else {
                    launch_stream<3, 5, 2, 1, false>(NGC_STREAM_ARGS);
                }
            } else if (sh.nv == 4) {
                switch (sh.waves) {
                    NGC_STREAM_CASE(4, 4, 1, true) NGC_STREAM_CASE(4, 4, 2, true)
                    NGC_STREAM_CASE(4, 4, 4, true)
                    NGC_STREAM_CASE(4, 4, 5, true) NGC_STREAM_CASE(4, 4, 6, true)
                    NGC_STREAM_CASE(4, 4, 7, true) NGC_STREAM_CASE(4, 4, 8, true)
                }
            } else if (sh.nv == 8) {
                switch (sh.waves) {
                    NGC_STREAM_CASE(8, 2, 5, true) NGC_STREAM_CASE(8, 2, 6, true)
                    NGC_STREAM_CASE(8, 2, 7, true) NGC_STREAM_CASE(8, 2, 8, true)
                    case 10: launch_stream<8, 1, 2, 10, true, v4f, true>(NGC_STREAM_ARGS); break;
                    case 12: launch_stream<8, 1, 2, 12, true, v4f, true>(NGC_STREAM_ARGS); break;
                    case 14: launch_stream<8, 1, 2, 14, true, v4f, true>(NGC_STREAM_ARGS); break;
                    case 16: launch_stream<8, 1, 2, 16, true, v4f, true>(NGC_STREAM_ARGS); break;
                }
            } else if (sh.nv == 1) {
                launch_stream<1, 16, 2, 1, true>(NGC_STREAM_ARGS);
            } else if (sh.nv == 2) {
                launch_stream<2, 8, 2, 1, true>(NGC_STREAM_ARGS);
            } else if (sh.waves == 4) {
                launch_stream<3, 5, 2, 4, true>(NGC_STREAM_ARGS);
            } else {
                launch_stream<3, 5, 2, 1, true>(NGC_STREAM_ARGS);
            }
#undef NGC_STREAM_ARGS
#undef NGC_STREAM_SCALAR
#undef NGC_STREAM_CASE
        }
        NGC_HIP(ctx, hipGetLastError());
        if (defer) {
            defer->ptr = ws;
            defer->chunks = (int)chunks;
            return NGC_OK;
        }
        {
            ngc_prof_scope ps(ctx, NGC_KERNEL_REDUCE);
            const int64_t dv = sh.scalar ? d : d / 4;
            dim3 grid((unsigned)((dv + 255) / 256), (unsigned)k);
            if (chunks >= 64) {  // short rows: many partials per partition, few columns
                dim3 grid64((unsigned)((dv + 63) / 64), (unsigned)k);
                if (sh.scalar)
                    hipLaunchKernelGGL((reduce_partials_deep_kernel<float>), grid64, dim3(64), 0, ctx->stream,
                                       (const float*)ws, G_dev, dv, (int)chunks, unit_row);
                else
                    hipLaunchKernelGGL((reduce_partials_deep_kernel<v4f>), grid64, dim3(64), 0, ctx->stream,
                                       (const v4f*)ws, (v4f*)G_dev, dv, (int)chunks, unit_row);
            } else if (sh.scalar)
                hipLaunchKernelGGL((reduce_partials_kernel<float>), grid, dim3(256), 0, ctx->stream,
                                   (const float*)ws, G_dev, dv, (int)chunks, unit_row);
            else
                hipLaunchKernelGGL((reduce_partials_kernel<v4f>), grid, dim3(256), 0, ctx->stream,
                                   (const v4f*)ws, (v4f*)G_dev, dv, (int)chunks, unit_row);
        }
        NGC_HIP(ctx, hipGetLastError());
        return NGC_OK;
    }
    // generic two-pass route
    const int64_t total_rows = (int64_t)k * rows;
    // float4 elements when rows and theta are 16-byte addressable (the partials always are: the
    // workspace is 256-byte aligned and the residuals before them take a multiple of 64 floats)
    const bool vec = d % 4 == 0 && ((reinterpret_cast<uintptr_t>(X_dev) | reinterpret_cast<uintptr_t>(theta_dev)) & 15) == 0;
    const int64_t dv = vec ? d / 4 : d;
    const int64_t col_blocks = (dv + 255) / 256;
    int64_t chunks = std::max<int64_t>(1, std::min<int64_t>(rows, (wave_slots / 4 + k * col_blocks - 1) / (k * col_blocks)));
    chunks = std::min<int64_t>(chunks, 65535);
    int64_t rpc = (rows + chunks - 1) / chunks;
    chunks = (rows + rpc - 1) / rpc;
    const size_t resid_floats = ((size_t)total_rows + 63) / 64 * 64;
    rc = get_ws(sizeof(float) * (resid_floats + (size_t)k * chunks * d));
    if (rc) return rc;
    float* resid = ws;
    float* partial = ws + resid_floats;
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_GRAD);
        const int64_t blocks = std::min<int64_t>((total_rows + 3) / 4, (int64_t)ctx->cu_count * 8);
#define NGC_RESID(LOSS_ID, VEC)                                                                                  \
    hipLaunchKernelGGL((resid_kernel<LOSS_ID, VEC>), dim3((unsigned)blocks), dim3(256), 0, ctx->stream, X_dev, y, \
                       theta_dev, resid, total_rows, d, rows, unit_part)
        if (loss == NGC_LOSS_LSQ) {
            if (vec) NGC_RESID(NGC_LOSS_LSQ, true); else NGC_RESID(NGC_LOSS_LSQ, false);
        } else {
            if (vec) NGC_RESID(NGC_LOSS_LOGISTIC, true); else NGC_RESID(NGC_LOSS_LOGISTIC, false);
        }
#undef NGC_RESID
        NGC_HIP(ctx, hipGetLastError());
        dim3 grid((unsigned)col_blocks, (unsigned)chunks, (unsigned)k);
        if (vec)
            hipLaunchKernelGGL(xtr_kernel<true>, grid, dim3(256), 0, ctx->stream, X_dev, resid, partial, rows, d,
                               (int)chunks, rpc, unit_part);
        else
            hipLaunchKernelGGL(xtr_kernel<false>, grid, dim3(256), 0, ctx->stream, X_dev, resid, partial, rows, d,
                               (int)chunks, rpc, unit_part);
    }
    NGC_HIP(ctx, hipGetLastError());
    if (defer) {
        defer->ptr = partial;
        defer->chunks = (int)chunks;
        return NGC_OK;
    }
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_REDUCE);
        dim3 grid((unsigned)((d + 255) / 256), (unsigned)k);
        hipLaunchKernelGGL((reduce_partials_kernel<float>), grid, dim3(256), 0, ctx->stream,
                           (const float*)partial, G_dev, d, (int)chunks, unit_row);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
}

extern "C" int ngc_partition_grads(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                                   const float* theta_dev, int64_t rows, float* G_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!X_dev || !y_dev || !theta_dev || !G_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null device pointer");
    if (rows < 1) return ngc_fail(ctx, NGC_ERR_INVALID, "rows_per_part must be positive");
    if (!ngc_aligned16(X_dev) || !ngc_aligned16(theta_dev) || !ngc_aligned16(G_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "X, theta and G must be 16-byte aligned");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    if (loss == NGC_LOSS_MLP2) {
        if (!ctx->mlp_din) return ngc_fail(ctx, NGC_ERR_STATE, "call ngc_set_mlp2_shape first");
        return ngc_mlp2_grads(ctx, X_dev, (const int*)y_dev, theta_dev, rows, G_dev, ctx->k, nullptr, nullptr);
    }
    if (loss != NGC_LOSS_LSQ && loss != NGC_LOSS_LOGISTIC) return ngc_fail(ctx, NGC_ERR_INVALID, "unknown loss");
    return grads_impl(ctx, loss, X_dev, y_dev, theta_dev, rows, G_dev, ctx->k, nullptr, nullptr);
} catch (...) {
    return ngc_on_exception();
}

// ---- partition gradients without any allocation ------------------------------------------
// The block partials of the gradient kernels go to a file-scope device array instead of the
// context's workspace.  Its name is only a host-side handle: the address a kernel can use is
// looked up once per device with hipGetSymbolAddress (each GPU holds its own copy of the array
// at its own address) and that pointer is what the launches get.
constexpr size_t NGC_STATIC_SCRATCH_BYTES = (size_t)20 << 20;
constexpr int NGC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[NGC_STATIC_SCRATCH_BYTES];
static float* static_scratch_ptr[NGC_MAX_DEVICES];  // per device, filled on the first call there
static std::mutex static_scratch_lock;

static int static_scratch(ngc_ctx* ctx, float** out) {
    int dev = -1;
    NGC_HIP(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= NGC_MAX_DEVICES) return ngc_fail(ctx, NGC_ERR_INVALID, "device index out of range");
    std::lock_guard<std::mutex> hold(static_scratch_lock);
    if (!static_scratch_ptr[dev]) {
        void* p = nullptr;
        NGC_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return ngc_fail(ctx, NGC_ERR_HIP, "hipGetSymbolAddress gave a null address");
        static_scratch_ptr[dev] = (float*)p;
    }
    *out = static_scratch_ptr[dev];
    return NGC_OK;
}

extern "C" int ngc_partition_grads_static(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                                          const float* theta_dev, int64_t rows, float* G_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!X_dev || !y_dev || !theta_dev || !G_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null device pointer");
    if (rows < 1) return ngc_fail(ctx, NGC_ERR_INVALID, "rows_per_part must be positive");
    if (!ngc_aligned16(X_dev) || !ngc_aligned16(theta_dev) || !ngc_aligned16(G_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "X, theta and G must be 16-byte aligned");
    if (loss == NGC_LOSS_MLP2)
        return ngc_fail(ctx, NGC_ERR_INVALID, "the perceptron's activations do not fit the static scratch");
    if (loss != NGC_LOSS_LSQ && loss != NGC_LOSS_LOGISTIC) return ngc_fail(ctx, NGC_ERR_INVALID, "unknown loss");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    float* ws = nullptr;
    rc = static_scratch(ctx, &ws);
    if (rc) return rc;
    // no event is created on this path: launches here are not recorded by the profiler
    const bool was = ctx->prof_suspended;
    ctx->prof_suspended = true;
    rc = grads_impl(ctx, loss, X_dev, y_dev, theta_dev, rows, G_dev, ctx->k, nullptr, nullptr, nullptr, ws,
                    NGC_STATIC_SCRATCH_BYTES);
    ctx->prof_suspended = was;
    return rc;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_update(ngc_ctx* ctx, float* theta_dev, const float* g_dev, double scale) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!theta_dev || !g_dev) return ngc_fail(ctx, NGC_ERR_INVALID, "null device pointer");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_UPDATE);
        hipLaunchKernelGGL(update_kernel, dim3((unsigned)((ctx->d + 255) / 256)), dim3(256), 0, ctx->stream,
                           theta_dev, g_dev, (float)scale, ctx->d);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---- measurement probes -----------------------------------------------------
extern "C" int ngc_probe_copy(ngc_ctx* ctx, const void* src_dev, void* dst_dev, int64_t bytes) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!src_dev || !dst_dev || bytes < 16 || bytes % 16 || !ngc_aligned16(src_dev) || !ngc_aligned16(dst_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "probe buffers must be 16-byte aligned, size a multiple of 16");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    const int64_t nvec = bytes / 16;
    const int64_t blocks = std::min<int64_t>((nvec + 255) / 256, (int64_t)ctx->cu_count * 16);
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_PROBE);
        hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                           (const v4f*)src_dev, (v4f*)dst_dev, nvec);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

extern "C" int ngc_probe_read(ngc_ctx* ctx, const void* src_dev, int64_t bytes) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!src_dev || bytes < 16 || bytes % 16 || !ngc_aligned16(src_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "probe buffer must be 16-byte aligned, size a multiple of 16");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    const int64_t nvec = bytes / 16;
    const int64_t blocks = std::min<int64_t>((nvec + 255) / 256, (int64_t)ctx->cu_count * 8);
    rc = ensure_ws(ctx, sizeof(float) * 4 * (size_t)blocks);
    if (rc) return rc;
    {
        ngc_prof_scope ps(ctx, NGC_KERNEL_PROBE);
        hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                           (const v4f*)src_dev, ctx->d_ws, nvec);
    }
    NGC_HIP(ctx, hipGetLastError());
    return NGC_OK;
} catch (...) {
    return ngc_on_exception();
}

// ---- redundancy-faithful worker execution ------------------------------------------------------
// room for `ints` map entries in both copies (device + pinned host staging)
static int ensure_maps(ngc_ctx* ctx, size_t ints) {
    if (ints <= ctx->maps_cap) return NGC_OK;
    NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (int q = 0; q < 2; ++q) {
        if (ctx->d_maps[q]) NGC_HIP(ctx, hipFree(ctx->d_maps[q]));
        if (ctx->h_maps[q]) NGC_HIP(ctx, hipHostFree(ctx->h_maps[q]));
        ctx->d_maps[q] = ctx->h_maps[q] = nullptr;
        ctx->maps_ev_set[q] = false;
    }
    ctx->maps_cap = 0;
    for (int q = 0; q < 2; ++q) {
        void* dp = nullptr;
        void* hp = nullptr;
        if (hipMalloc(&dp, ints * sizeof(int)) != hipSuccess || hipHostMalloc(&hp, ints * sizeof(int)) != hipSuccess) {
            (void)hipGetLastError();
            if (dp) (void)hipFree(dp);
            return ngc_fail(ctx, NGC_ERR_NOMEM, "map allocation failed");
        }
        ctx->d_maps[q] = (int*)dp;
        ctx->h_maps[q] = (int*)hp;
        if (!ctx->maps_ev[q]) NGC_HIP(ctx, hipEventCreateWithFlags(&ctx->maps_ev[q], hipEventDisableTiming));
    }
    ctx->maps_cap = ints;
    return NGC_OK;
}

extern "C" int ngc_worker_grads(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                                const float* theta_dev, int64_t rows, const int* progress_host,
                                float* W_dev) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!X_dev || !y_dev || !theta_dev || !W_dev || !progress_host) return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (rows < 1) return ngc_fail(ctx, NGC_ERR_INVALID, "rows_per_part must be positive");
    if (loss != NGC_LOSS_LSQ && loss != NGC_LOSS_LOGISTIC && loss != NGC_LOSS_MLP2)
        return ngc_fail(ctx, NGC_ERR_INVALID, "unknown loss");
    if (loss == NGC_LOSS_MLP2 && !ctx->mlp_din) return ngc_fail(ctx, NGC_ERR_STATE, "call ngc_set_mlp2_shape first");
    if (!ngc_aligned16(X_dev) || !ngc_aligned16(theta_dev) || !ngc_aligned16(W_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "X, theta and W must be 16-byte aligned");
    int rc = ngc_dev_init(ctx);
    if (rc) return rc;
    ngc_worker_plan plan;
    rc = ngc_make_worker_plan(ctx, plan);
    if (rc) return rc;
    const int n = ctx->n, Tp = plan.T * ctx->c;  // partitions per worker schedule
    std::vector<int> part, row;
    for (int i = 0; i < n; ++i) {
        if (progress_host[i] < 0) return ngc_fail(ctx, NGC_ERR_INVALID, "negative progress");
        const int64_t want = (int64_t)progress_host[i] * ctx->c;  // c partitions per finished task
        const int done = (int)std::min<int64_t>(want, (int64_t)plan.order[i].size());
        for (int t = 0; t < done; ++t) {
            part.push_back(plan.order[i][t]);
            row.push_back(i * Tp + t);
        }
    }
    const int units = (int)part.size();
    if (units == 0) return NGC_OK;
    rc = ensure_maps(ctx, (size_t)2 * n * Tp);
    if (rc) return rc;
    // maps: unit_part | unit_row.  The copy used two calls ago is free once its kernels are done.
    const int q = ctx->maps_turn ^= 1;
    if (ctx->maps_ev_set[q]) NGC_HIP(ctx, hipEventSynchronize(ctx->maps_ev[q]));
    std::memcpy(ctx->h_maps[q], part.data(), sizeof(int) * units);
    std::memcpy(ctx->h_maps[q] + units, row.data(), sizeof(int) * units);
    NGC_HIP(ctx, hipMemcpyAsync(ctx->d_maps[q], ctx->h_maps[q], sizeof(int) * 2 * units, hipMemcpyHostToDevice,
                                ctx->stream));
    if (loss == NGC_LOSS_MLP2)
        rc = ngc_mlp2_grads(ctx, X_dev, (const int*)y_dev, theta_dev, rows, W_dev, units, ctx->d_maps[q],
                            ctx->d_maps[q] + units);
    else
        rc = grads_impl(ctx, loss, X_dev, y_dev, theta_dev, rows, W_dev, units, ctx->d_maps[q],
                        ctx->d_maps[q] + units);
    NGC_HIP(ctx, hipEventRecord(ctx->maps_ev[q], ctx->stream));
    ctx->maps_ev_set[q] = true;
    return rc;
} catch (...) {
    return ngc_on_exception();
}

// ---- one whole iteration in two launches ----------------------------------------------------------
extern "C" int ngc_iteration(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                             float* theta_dev, int64_t rows, const uint8_t* straggler_mask,
                             double scale, float* G_dev, float* C_dev, float* g_dev, int* layer_out,
                             double* a_out) try {
    if (!ctx) return NGC_ERR_INVALID;
    if (!X_dev || !y_dev || !theta_dev || !G_dev || !C_dev || !g_dev || !straggler_mask)
        return ngc_fail(ctx, NGC_ERR_INVALID, "null pointer");
    if (rows < 1) return ngc_fail(ctx, NGC_ERR_INVALID, "rows_per_part must be positive");
    if (loss != NGC_LOSS_LSQ && loss != NGC_LOSS_LOGISTIC && loss != NGC_LOSS_MLP2)
        return ngc_fail(ctx, NGC_ERR_INVALID, "unknown loss");
    if (!ngc_aligned16(X_dev) || !ngc_aligned16(theta_dev) || !ngc_aligned16(G_dev) || !ngc_aligned16(C_dev) || !ngc_aligned16(g_dev))
        return ngc_fail(ctx, NGC_ERR_INVALID, "device buffers must be 16-byte aligned");
    // main-node bookkeeping first: an undecodable round launches nothing
    double a[NGC_MAX_N];
    int layer = -1;
    double resid = 0.0;
    int rc = ngc_select_decode_vec(ctx, straggler_mask, &layer, a, &resid);
    if (layer_out) *layer_out = layer;
    if (rc) return rc;
    if (a_out) std::memcpy(a_out, a, sizeof(double) * ctx->n);
    if (loss == NGC_LOSS_MLP2) {  // no block partials to fuse: the stand-alone calls in sequence
        rc = ngc_partition_grads(ctx, loss, X_dev, y_dev, theta_dev, rows, G_dev);
        if (!rc) rc = ngc_encode(ctx, G_dev, -1, C_dev);
        if (!rc) rc = ngc_decode(ctx, layer, a, C_dev, g_dev);
        if (!rc) rc = ngc_update(ctx, theta_dev, g_dev, scale);
        return rc;
    }
    rc = ngc_dev_init(ctx);
    if (rc) return rc;
    partial_info pi;
    rc = grads_impl(ctx, loss, X_dev, y_dev, theta_dev, rows, G_dev, ctx->k, nullptr, nullptr, &pi);
    if (rc) return rc;
    return ngc_launch_tail(ctx, pi.ptr, pi.chunks, layer, a, G_dev, C_dev, g_dev, theta_dev, scale);
} catch (...) {
    return ngc_on_exception();
}
