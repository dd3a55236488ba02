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

// ---------------------------------------------------------------------------
// wave-wide sum, result in every lane.  Four DPP steps give each row of 16
// lanes its own sum; the four row sums are then added in a fixed order.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_step(float v) {
    int iv = __builtin_bit_cast(int, v);
    int sh = __builtin_amdgcn_update_dpp(iv, iv, CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, sh);
}

__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_step<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_step<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_step<0x141>(v);  // row_half_mirror
    v = dpp_step<0x140>(v);  // row_mirror
    int iv = __builtin_bit_cast(int, v);
    float s0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    float s1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    float s2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    float s3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return (s0 + s1) + (s2 + s3);
}

// d/dz of the per-sample loss at margin z = x.theta (the factor of x in the gradient)
template <int LOSS>
__device__ __forceinline__ float loss_slope(float z, float y) {
    if (LOSS == NGC_LOSS_LSQ) return z - y;
    // logistic, labels +/-1:  -y / (1 + exp(y z)); exp overflow gives the correct limit 0
    return -y / (1.0f + expf(y * z));
}

// ---------------------------------------------------------------------------
// K1: single-pass partition gradient for d = WAVES * 256 * NV.
// A block of WAVES waves owns a run of consecutive rows of one partition; wave w
// owns columns [w*256*NV, (w+1)*256*NV) of every row.  A group of R rows sits in
// registers (lane l holds float4 number i*64+l of the wave's slice, i < NV), so
// the same registers feed the dot product x.theta and, once the residual is
// known, the update acc += r*x: X is read from HBM exactly once.  While a group
// is consumed the following NBUF-1 groups are already in flight.  The waves
// exchange their partial dot products through LDS, one barrier per group; the
// exchange area is double buffered so a fast wave cannot overwrite values a
// slow wave still has to read.  theta and the accumulator stay in registers.
// Each block writes one partial sum per partition run; K2 adds them in a fixed
// order.
// ---------------------------------------------------------------------------
template <int NV, int R, typename VT>
struct row_group {
    VT x[R][NV];
    float y;  // lane l < R holds the label of row l of the group
};

// The lane's i-th element (a float4, or a float when rows are not 16-byte
// aligned) sits lane_off + i*64 elements into the row, `pitch` is the row length
// in bytes.  For the exact shapes lane_off counts from the wave's slice and the
// rest are compile-time constants; for ragged rows (RAGGED) lane_off counts
// from the row's start and offsets past `last_off`, the row's last element,
// are clamped to it.
template <int NV, int R, int DV, bool RAGGED, typename VT>
__device__ __forceinline__ void load_group(row_group<NV, R, VT>& b, const char* __restrict__ xbase,
                                           const float* __restrict__ yp, uint32_t lane_off,
                                           uint32_t last_off, int64_t pitch, int lane,
                                           int64_t row, int64_t last_row) {
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        int64_t r = row + rr;
        r = r < last_row ? r : last_row;  // past the end: re-read the last row; its weight is 0
        const char* p = xbase + r * (RAGGED ? pitch : (int64_t)(DV * sizeof(VT)));  // wave-uniform
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            uint32_t o = lane_off + i * 64 * (int)sizeof(VT);
            if (RAGGED) o = o < last_off ? o : last_off;
            b.x[rr][i] = __builtin_nontemporal_load(reinterpret_cast<const VT*>(p + o));
        }
    }
    int64_t ry = row + (lane < R ? lane : R - 1);
    ry = ry < last_row ? ry : last_row;
    b.y = yp[ry];
}

__device__ __forceinline__ float hsum(float q) { return q; }
__device__ __forceinline__ float hsum(v4f q) { return (q.x + q.y) + (q.z + q.w); }

template <int NV, int R, int WAVES, int LOSS, typename VT>
__device__ __forceinline__ void consume_group(const row_group<NV, R, VT>& b, VT (&acc)[NV],
                                              const VT (&th)[NV], float* ex, int wave,
                                              int lane, int64_t row, int64_t end_row) {
    float dot[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        VT q = b.x[rr][0] * th[0];
#pragma unroll
        for (int i = 1; i < NV; ++i) q += b.x[rr][i] * th[i];
        dot[rr] = wave_sum(hsum(q));
    }
    if (WAVES > 1) {
        // ex[rr*WAVES + w]: every lane of wave w stores the same value
#pragma unroll
        for (int rr = 0; rr < R; ++rr) ex[rr * WAVES + wave] = dot[rr];
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            float z = ex[rr * WAVES];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) z += ex[rr * WAVES + w];
            dot[rr] = z;
        }
    }
    if (LOSS == NGC_LOSS_LSQ) {
        const int yi = __builtin_bit_cast(int, b.y);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            float yv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(yi, rr));
            float res = (row + rr < end_row) ? loss_slope<LOSS>(dot[rr], yv) : 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] += res * b.x[rr][i];
        }
    } else {
        // The slope costs an exponential and a division.  The R margins of the
        // group are wave-uniform, so lane l takes the margin of row l (its label is
        // already there) and the slopes of all R rows come out of one pass; each is
        // then broadcast from its lane.  Rows past the end get weight 0 as a factor
        // (the re-read row's slope is finite), which keeps the loop body free of
        // branches.
        float zv = 0.0f;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) zv = (lane == rr) ? dot[rr] : zv;
        const float live = (row + lane < end_row) ? 1.0f : 0.0f;
        const int sv = __builtin_bit_cast(int, loss_slope<LOSS>(zv, b.y) * live);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            float res = __builtin_bit_cast(float, __builtin_amdgcn_readlane(sv, rr));
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] += res * b.x[rr][i];
        }
    }
}

template <int NV, int R, int NBUF, int WAVES, int LOSS, bool RAGGED, typename VT>
__global__ __launch_bounds__(WAVES * 64) void grad_stream_kernel(
    const float* __restrict__ X, const float* __restrict__ y, const float* __restrict__ theta,
    float* __restrict__ partial, int64_t rows, int chunks, int64_t rows_per_chunk,
    const int* __restrict__ unit_part, int dq) {
    // elements (VT: float4, or float for rows that are not 16-byte aligned) per
    // row: the block's WAVES*64*NV slots for the exact shapes; for ragged rows the
    // true count dq (<= the slots), slots past it are idle: they re-read the
    // row's last element against a zero of theta and store nothing
    constexpr int SLOTS = WAVES * 64 * NV;
    const int64_t dv = RAGGED ? dq : SLOTS;
    __shared__ float ex_s[2][R * WAVES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // a unit is one partial-gradient computation; by default unit j is partition j,
    // with unit_part several units may work on the same partition (one per worker)
    const int unit = blockIdx.x / chunks;
    const int j = unit_part ? unit_part[unit] : unit;
    const int c = blockIdx.x % chunks;
    const int64_t r0 = (int64_t)c * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const char* xbase = reinterpret_cast<const char*>(X) +
                        ((int64_t)j * rows * dv + (RAGGED ? 0 : (int64_t)wave * 64 * NV)) * (int64_t)sizeof(VT);
    const float* yp = y + (int64_t)j * rows;
    const uint32_t lane_off =
        (uint32_t)((RAGGED ? wave * 64 * NV : 0) + lane) * (uint32_t)sizeof(VT);
    const uint32_t last_off = (uint32_t)(dv - 1) * (uint32_t)sizeof(VT);
    const int64_t pitch = dv * (int64_t)sizeof(VT);

    VT th[NV], acc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int slot = wave * 64 * NV + i * 64 + lane;
        if (RAGGED)
            th[i] = slot < dq ? reinterpret_cast<const VT*>(theta)[slot] : (VT)(0.0f);
        else
            th[i] = reinterpret_cast<const VT*>(theta)[slot];
        acc[i] = (VT)(0.0f);
    }

    // Groups are taken NBUF at a time with no branch inside the loop, so that the
    // waits the compiler places before a group's first use cover only that
    // group's loads and leave the younger ones in flight.  Groups past the end of
    // the run re-read its last row (a cache hit) and get weight 0.
    const int64_t ngroups = r0 < r1 ? (r1 - r0 + R - 1) / R : 0;  // block-uniform
    if (ngroups > 0) {
        const int64_t last = r1 - 1;
        row_group<NV, R, VT> buf[NBUF];
#pragma unroll
        for (int p = 0; p < NBUF - 1; ++p)
            load_group<NV, R, SLOTS, RAGGED, VT>(buf[p], xbase, yp, lane_off, last_off, pitch, lane,
                                             r0 + (int64_t)p * R, last);
        for (int64_t gb = 0; gb < ngroups; gb += NBUF) {
#pragma unroll
            for (int p = 0; p < NBUF; ++p) {
                const int64_t gi = gb + p;
                load_group<NV, R, SLOTS, RAGGED, VT>(buf[(p + NBUF - 1) % NBUF], xbase, yp, lane_off,
                                                     last_off, pitch, lane, r0 + (gi + NBUF - 1) * R, last);
                consume_group<NV, R, WAVES, LOSS, VT>(buf[p], acc, th, ex_s[gi & 1], wave, lane, r0 + gi * R, r1);
            }
        }
    }
    VT* out = reinterpret_cast<VT*>(partial) + (int64_t)blockIdx.x * dv;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int slot = wave * 64 * NV + i * 64 + lane;
        if (!RAGGED || slot < dq) out[slot] = acc[i];
    }
}

// ---------------------------------------------------------------------------
// Single-pass partition gradient for narrow rows: d = 4*DQ with DQ = 1, 2, 4, .. 32 float4 per
// row (4 to 128 features).  Rows are contiguous in memory, so one wave-wide 16-byte load
// (1 KiB) fetches RPL = 64/DQ whole rows: lane l holds float4 number l % DQ of row l / DQ.
// The dot product of a row is a sum over its DQ lanes (DPP steps inside a row of 16 lanes, one
// cross-lane exchange for 32), after which every lane of the segment knows its row's slope and
// adds slope * x into its own accumulator; the accumulators of the RPL segments are added once,
// at the end, through LDS in segment order.  R loads form a group, the next group is in
// flight while one is consumed; rows past the end re-read the last row with weight 0.  One
// wave per block.
// ---------------------------------------------------------------------------
template <int DQ>
__device__ __forceinline__ float segment_sum(float v) {
    if (DQ >= 2) v = dpp_step<0xB1>(v);   // quad_perm [1,0,3,2]
    if (DQ >= 4) v = dpp_step<0x4E>(v);   // quad_perm [2,3,0,1]
    if (DQ >= 8) v = dpp_step<0x141>(v);  // row_half_mirror
    if (DQ >= 16) v = dpp_step<0x140>(v); // row_mirror
    if (DQ >= 32) v += __shfl_xor(v, 16);
    return v;
}

template <int R>
struct narrow_group {
    v4f x[R];
    float y[R];
};

template <int DQ, int R>
__device__ __forceinline__ void load_narrow(narrow_group<R>& b, const v4f* __restrict__ xp,
                                            const float* __restrict__ yp, int seg, int slot,
                                            int64_t row, int64_t last_row) {
    constexpr int RPL = 64 / DQ;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        int64_t r = row + u * RPL + seg;
        r = r < last_row ? r : last_row;
        b.x[u] = __builtin_nontemporal_load(xp + r * DQ + slot);
        b.y[u] = yp[r];
    }
}

template <int DQ, int R, int LOSS>
__device__ __forceinline__ void consume_narrow(const narrow_group<R>& b, v4f& acc, const v4f th, int seg,
                                               int64_t row, int64_t end_row) {
    constexpr int RPL = 64 / DQ;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const float z = segment_sum<DQ>(hsum(b.x[u] * th));
        const float live = (row + u * RPL + seg < end_row) ? 1.0f : 0.0f;
        const float res = loss_slope<LOSS>(z, b.y[u]) * live;
        acc += res * b.x[u];
    }
}

template <int DQ, int R, int LOSS>
__global__ __launch_bounds__(64) void grad_narrow_kernel(const float* __restrict__ X, const float* __restrict__ y,
                                                         const float* __restrict__ theta,
                                                         float* __restrict__ partial, int64_t rows, int chunks,
                                                         int64_t rows_per_chunk,
                                                         const int* __restrict__ unit_part) {
    constexpr int RPL = 64 / DQ;
    __shared__ v4f red[64];
    const int lane = threadIdx.x;
    const int seg = lane / DQ, slot = lane % DQ;
    const int unit = blockIdx.x / chunks;
    const int j = unit_part ? unit_part[unit] : unit;
    const int c = blockIdx.x % chunks;
    const int64_t r0 = (int64_t)c * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const v4f* xp = reinterpret_cast<const v4f*>(X) + (int64_t)j * rows * DQ;
    const float* yp = y + (int64_t)j * rows;
    const v4f th = reinterpret_cast<const v4f*>(theta)[slot];
    v4f acc = (v4f)(0.0f);
    constexpr int GROUP = R * RPL;  // rows per group
    const int64_t ngroups = r0 < r1 ? (r1 - r0 + GROUP - 1) / GROUP : 0;
    if (ngroups > 0) {
        const int64_t last = r1 - 1;
        narrow_group<R> buf[2];
        load_narrow<DQ, R>(buf[0], xp, yp, seg, slot, r0, last);
        for (int64_t gb = 0; gb < ngroups; gb += 2) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int64_t gi = gb + p;
                load_narrow<DQ, R>(buf[(p + 1) % 2], xp, yp, seg, slot, r0 + (gi + 1) * GROUP, last);
                consume_narrow<DQ, R, LOSS>(buf[p], acc, th, seg, r0 + gi * GROUP, r1);
            }
        }
    }
    red[lane] = acc;
    __syncthreads();
    if (lane < DQ) {
        v4f s = red[lane];
#pragma unroll
        for (int g = 1; g < RPL; ++g) s += red[g * DQ + lane];
        reinterpret_cast<v4f*>(partial)[(int64_t)blockIdx.x * DQ + lane] = s;
    }
}

// ---------------------------------------------------------------------------
// Generic two-pass route for any d.  Pass 1: one wave per row forms the margin
// and stores the residual.  Pass 2: one thread per column adds r*x over a run
// of rows; partials are summed by K2.
// ---------------------------------------------------------------------------
template <int LOSS>
__global__ __launch_bounds__(256) void resid_kernel(const float* __restrict__ X,
                                                    const float* __restrict__ y,
                                                    const float* __restrict__ theta,
                                                    float* __restrict__ resid, int64_t total_rows,
                                                    int64_t d, int64_t rows,
                                                    const int* __restrict__ unit_part) {
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t r = wave0; r < total_rows; r += nwaves) {
        // row r of the unit list is row (r % rows) of partition unit_part[r / rows]
        const int64_t src = unit_part ? (int64_t)unit_part[r / rows] * rows + r % rows : r;
        const float* xr = X + src * d;
        float dot = 0.0f;
        for (int64_t c = lane; c < d; c += 64) dot += xr[c] * theta[c];
        float z = wave_sum(dot);
        if (lane == 0) resid[r] = loss_slope<LOSS>(z, y[src]);
    }
}

__global__ __launch_bounds__(256) void xtr_kernel(const float* __restrict__ X,
                                                  const float* __restrict__ resid,
                                                  float* __restrict__ partial, int64_t rows,
                                                  int64_t d, int chunks, int64_t rows_per_chunk,
                                                  const int* __restrict__ unit_part) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y;
    const int j = blockIdx.z;  // unit
    if (c >= d) return;
    const int64_t r0 = (int64_t)chunk * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const int part = unit_part ? unit_part[j] : j;
    const float* xp = X + ((int64_t)part * rows) * d + c;
    const float* rp = resid + (int64_t)j * rows;
    float acc = 0.0f;
    for (int64_t r = r0; r < r1; ++r) acc += rp[r] * xp[r * d];
    partial[((int64_t)j * chunks + chunk) * d + c] = acc;
}

// K2: G[j][:] = sum over chunks of partial[j][chunk][:], chunks added in index order.
template <typename VT>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const VT* __restrict__ partial,
                                                              VT* __restrict__ G, int64_t dv,
                                                              int chunks,
                                                              const int* __restrict__ unit_row) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int j = blockIdx.y;
    if (c >= dv) return;
    const VT* p = partial + (int64_t)j * chunks * dv + c;
    VT acc = p[0];
    int t = 1;
    for (; t + 4 <= chunks; t += 4) {
        VT a0 = p[(int64_t)t * dv], a1 = p[(int64_t)(t + 1) * dv];
        VT a2 = p[(int64_t)(t + 2) * dv], a3 = p[(int64_t)(t + 3) * dv];
        acc = (((acc + a0) + a1) + a2) + a3;
    }
    for (; t < chunks; ++t) acc += p[(int64_t)t * dv];
    G[(int64_t)(unit_row ? unit_row[j] : j) * dv + c] = acc;
}

// K6: theta -= scale * g
__global__ __launch_bounds__(256) void update_kernel(float* __restrict__ theta,
                                                     const float* __restrict__ g, float scale,
                                                     int64_t d) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c < d) theta[c] = theta[c] - scale * g[c];
}

// ---------------------------------------------------------------------------
// Measurement probes (not part of the method): a plain copy and a plain read of
// a known number of bytes, used to calibrate HBM byte counters and to find the
// read bandwidth a trivial kernel reaches on the same buffers.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_copy_kernel(const v4f* __restrict__ src,
                                                         v4f* __restrict__ dst, int64_t nvec) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride)
        dst[i] = __builtin_nontemporal_load(src + i);
}

__global__ __launch_bounds__(256) void probe_read_kernel(const v4f* __restrict__ src,
                                                         float* __restrict__ sink, int64_t nvec) {
    // every block reads a contiguous run, 8 independent 16-byte loads per thread in flight
    const int64_t per_block = (nvec + gridDim.x - 1) / gridDim.x;
    const int64_t b0 = (int64_t)blockIdx.x * per_block;
    const int64_t b1 = b0 + per_block < nvec ? b0 + per_block : nvec;
    v4f acc = (v4f)(0.0f);
    int64_t i = b0 + threadIdx.x;
    for (; i + 7 * 256 < b1; i += 8 * 256) {
        v4f t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += t[u];
    }
    for (; i < b1; i += 256) acc += __builtin_nontemporal_load(src + i);
    float s = wave_sum((acc.x + acc.y) + (acc.z + acc.w));
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
}


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
template <int NV, int R, int NBUF, int WAVES, bool RAGGED, typename VT = v4f>
static void launch_stream(ngc_ctx* ctx, int loss, const float* X, const float* y,
                          const float* theta, float* partial, int k, int64_t rows, int chunks,
                          int64_t rpc, const int* unit_part, int dq) {
    dim3 grid((unsigned)(k * chunks));
    if (loss == NGC_LOSS_LSQ)
        hipLaunchKernelGGL((grad_stream_kernel<NV, R, NBUF, WAVES, NGC_LOSS_LSQ, RAGGED, VT>), grid,
                           dim3(WAVES * 64), 0, ctx->stream, X, y, theta, partial, rows, chunks, rpc,
                           unit_part, dq);
    else
        hipLaunchKernelGGL((grad_stream_kernel<NV, R, NBUF, WAVES, NGC_LOSS_LOGISTIC, RAGGED, VT>), grid,
                           dim3(WAVES * 64), 0, ctx->stream, X, y, theta, partial, rows, chunks, rpc,
                           unit_part, dq);
}

// Shape of the single-pass kernel for a given d, or waves = 0 if d has none
// (above 16384, or above 8192 and not a multiple of 4).  A block offers
// nv*waves*64 slots per row, each a float4, or a float (`scalar`) when d is not
// a multiple of 4 and rows are therefore not 16-byte aligned; `ragged` when
// the row has fewer elements than the block has slots.
struct stream_shape {
    int nv, r, waves;
    bool ragged, scalar;
    int narrow_dq = 0;  // > 0: rows of narrow_dq float4 take grad_narrow_kernel (several rows per load)
};
static stream_shape pick_stream_shape(int64_t d) {
    if (d % 4 == 0 && d <= 128 && ((d / 4) & (d / 4 - 1)) == 0) return {1, 8, 1, false, false, (int)(d / 4)};
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
    if (d < 1 || d > 16384) return {0, 0, 0, false, false};
    if (d % 4 != 0) {
        if (d <= 256) return {4, 16, 1, true, true};
        if (d <= 4096) return {8, 8, (int)((d + 511) / 512), true, true};
        if (d <= 8192) return {16, 3, (int)((d + 1023) / 1024), true, true};
        return {0, 0, 0, false, false};
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

    const stream_shape sh = pick_stream_shape(d);
    if (sh.waves) {
        // enough blocks to give every SIMD two waves, split evenly over the partitions
        // a CU holds 8 such waves (2 per SIMD at up to 256 registers), so it takes
        // 8 / waves whole blocks; more blocks than that would run as a second,
        // partly filled round
        // rows of at most 128 features fill no more than half of a wave's lanes: twice the
        // blocks keep as many bytes in flight (measured: 3.1 -> 3.6 TB/s at 64 features,
        // 4.3 -> 5.0 at 100, 5.5 -> 6.1 at 128; wider rows lose 2 % with more than 8)
        const int per_cu = (sh.waves == 1 && !sh.scalar && d <= 128) ? 16 : std::max(1, 8 / sh.waves);
        const int64_t block_slots = (int64_t)ctx->cu_count * per_cu;
        int64_t chunks = std::max<int64_t>(1, block_slots / k);
        int64_t rpc = (rows + chunks - 1) / chunks;
        // two row groups: one trip of the kernel's loop (a narrow-row group is r loads of 64/dq rows)
        const int64_t quantum = sh.narrow_dq ? 2 * sh.r * (64 / sh.narrow_dq) : 2 * sh.r;
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
            if (sh.narrow_dq) {
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
            if (sh.scalar)
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
    const int64_t col_blocks = (d + 255) / 256;
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
        if (loss == NGC_LOSS_LSQ)
            hipLaunchKernelGGL((resid_kernel<NGC_LOSS_LSQ>), dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                               X_dev, y, theta_dev, resid, total_rows, d, rows, unit_part);
        else
            hipLaunchKernelGGL((resid_kernel<NGC_LOSS_LOGISTIC>), dim3((unsigned)blocks), dim3(256), 0,
                               ctx->stream, X_dev, y, theta_dev, resid, total_rows, d, rows, unit_part);
        NGC_HIP(ctx, hipGetLastError());
        dim3 grid((unsigned)col_blocks, (unsigned)chunks, (unsigned)k);
        hipLaunchKernelGGL(xtr_kernel, grid, dim3(256), 0, ctx->stream, X_dev, resid, partial, rows, d,
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
