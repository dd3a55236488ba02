// Device code of the partition-gradient path of libngc for gfx950 (CDNA4, wave64): the
// single-pass gradient kernels, the two-pass route, the fixed-order sum of block partials, the
// descent update and the measurement probes; the launchers are in ngc_device.hip.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

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

// th_l (TH_LDS): the lane's theta elements in LDS, element i at th_l[i * 64], instead of th.
template <int NV, int R, int WAVES, int LOSS, typename VT, bool TH_LDS = false>
__device__ __forceinline__ void consume_group(const row_group<NV, R, VT>& b, VT (&acc)[NV],
                                              const VT (&th)[TH_LDS ? 1 : NV], const VT* th_l, float* ex,
                                              int wave, int lane, int64_t row, int64_t end_row) {
    float dot[R];
    if (TH_LDS) {
        VT q[R];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const VT t = th_l[i * 64];
#pragma unroll
            for (int rr = 0; rr < R; ++rr) q[rr] = i == 0 ? b.x[rr][0] * t : q[rr] + b.x[rr][i] * t;
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) dot[rr] = wave_sum(hsum(q[rr]));
    } else {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            VT q = b.x[rr][0] * th[0];
#pragma unroll
            for (int i = 1; i < NV; ++i) q += b.x[rr][i] * th[i];
            dot[rr] = wave_sum(hsum(q));
        }
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

// TH_LDS: theta sits in LDS (one copy per block, each wave reads its own slice once per row
// group) instead of in registers; a wave with eight float4 per lane and row then stays within
// 128 registers, sixteen such waves form a block, and rows of up to 32768 features take one pass.
template <int NV, int R, int NBUF, int WAVES, int LOSS, bool RAGGED, typename VT, bool TH_LDS = false>
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

    __shared__ VT th_s[TH_LDS ? SLOTS : 1];
    VT th[TH_LDS ? 1 : NV], acc[NV];
    // the lane's elements of theta; with TH_LDS a wave writes and later reads only its own
    // slice, so no barrier is needed between the two
    const VT* th_l = th_s + (TH_LDS ? wave * 64 * NV + lane : 0);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int slot = wave * 64 * NV + i * 64 + lane;
        VT t;
        if (RAGGED)
            t = slot < dq ? reinterpret_cast<const VT*>(theta)[slot] : (VT)(0.0f);
        else
            t = reinterpret_cast<const VT*>(theta)[slot];
        if (TH_LDS)
            th_s[slot] = t;
        else
            th[i] = t;
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
                consume_group<NV, R, WAVES, LOSS, VT, TH_LDS>(buf[p], acc, th, th_l, ex_s[gi & 1], wave, lane, r0 + gi * R, r1);
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
// The same for any short row: dq elements per row (float4 when the rows are 16-byte aligned,
// dq <= 32; single floats otherwise, dq <= 32), known at run time.  A wave-wide load fetches
// rpl = 64 / dq whole rows (the lanes past rpl * dq idle: they re-read valid data against a
// zero of theta and a weight of 0); lane l holds element l % dq of row l / dq.  A row's dot
// product is a sum over dq consecutive lanes, folded in halves through the cross-lane shuffle
// (the part past the largest power of two below dq first, then 16, 8, .. 1: a fixed order) and
// handed back to every lane of the segment from its first lane.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float segment_sum_any(float v, int slot, int seg_base, int dq) {
    int len = dq;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        if (off < len) {  // wave-uniform
            const float t = __shfl_down(v, off, 64);
            if (slot + off < len) v += t;
            len = off;
        }
    }
    return __shfl(v, seg_base, 64);
}

template <typename VT, int R>
struct narrow_any_group {
    VT x[R];
    float y[R];
};

template <typename VT, int R>
__device__ __forceinline__ void load_narrow_any(narrow_any_group<VT, R>& b, const VT* __restrict__ xp,
                                                const float* __restrict__ yp, int seg, int slot, int dq, int rpl,
                                                int64_t row, int64_t last_row) {
#pragma unroll
    for (int u = 0; u < R; ++u) {
        int64_t r = row + u * rpl + seg;
        r = r < last_row ? r : last_row;
        b.x[u] = __builtin_nontemporal_load(xp + r * dq + slot);
        b.y[u] = yp[r];
    }
}

template <typename VT, int R, int LOSS>
__global__ __launch_bounds__(64) void grad_narrow_any_kernel(const float* __restrict__ X, const float* __restrict__ y,
                                                             const float* __restrict__ theta,
                                                             float* __restrict__ partial, int64_t rows, int chunks,
                                                             int64_t rows_per_chunk,
                                                             const int* __restrict__ unit_part, int dq) {
    __shared__ VT red[64];
    const int lane = threadIdx.x;
    const int rpl = 64 / dq;
    // lanes past the last whole row form a segment of their own (seg == rpl) that counts for nothing
    const int seg = lane / dq, slot = lane - seg * dq;
    const bool act = seg < rpl;
    const int unit = blockIdx.x / chunks;
    const int j = unit_part ? unit_part[unit] : unit;
    const int c = blockIdx.x % chunks;
    const int64_t r0 = (int64_t)c * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const VT* xp = reinterpret_cast<const VT*>(X) + (int64_t)j * rows * dq;
    const float* yp = y + (int64_t)j * rows;
    const VT th = act ? reinterpret_cast<const VT*>(theta)[slot] : (VT)(0.0f);
    VT acc = (VT)(0.0f);
    const int group = R * rpl;  // rows per group
    const int64_t ngroups = r0 < r1 ? (r1 - r0 + group - 1) / group : 0;
    if (ngroups > 0) {
        const int64_t last = r1 - 1;
        narrow_any_group<VT, R> buf[2];
        load_narrow_any<VT, R>(buf[0], xp, yp, seg, slot, dq, rpl, r0, last);
        for (int64_t gb = 0; gb < ngroups; gb += 2) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int64_t gi = gb + p;
                load_narrow_any<VT, R>(buf[(p + 1) % 2], xp, yp, seg, slot, dq, rpl, r0 + (gi + 1) * group, last);
                const int64_t row = r0 + gi * group;
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const float z = segment_sum_any(hsum(buf[p].x[u] * th), slot, seg * dq, dq);
                    const float live = (act && row + u * rpl + seg < r1) ? 1.0f : 0.0f;
                    const float res = loss_slope<LOSS>(z, buf[p].y[u]) * live;
                    acc += res * buf[p].x[u];
                }
            }
        }
    }
    red[lane] = acc;
    __syncthreads();
    if (lane < dq) {
        VT s = red[lane];
        for (int g = 1; g < rpl; ++g) s += red[g * dq + lane];
        reinterpret_cast<VT*>(partial)[(int64_t)blockIdx.x * dq + lane] = s;
    }
}

// ---------------------------------------------------------------------------
// Generic two-pass route for any d.  Pass 1: one wave per row forms the margin
// and stores the residual.  Pass 2: a thread adds r*x over a run of rows for its
// columns; partials are summed by K2.  VEC (d a multiple of 4, X 16-byte
// aligned): elements are float4.  Both passes keep eight loads per lane in flight;
// a column's terms are added in row order whatever the width.
// ---------------------------------------------------------------------------
template <int LOSS, bool VEC>
__global__ __launch_bounds__(256) void resid_kernel(const float* __restrict__ X,
                                                    const float* __restrict__ y,
                                                    const float* __restrict__ theta,
                                                    float* __restrict__ resid, int64_t total_rows,
                                                    int64_t d, int64_t rows,
                                                    const int* __restrict__ unit_part) {
    using VT = typename std::conditional<VEC, v4f, float>::type;
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t dv = VEC ? d / 4 : d;
    const VT* tv = reinterpret_cast<const VT*>(theta);
    for (int64_t r = wave0; r < total_rows; r += nwaves) {
        // row r of the unit list is row (r % rows) of partition unit_part[r / rows]
        const int64_t src = unit_part ? (int64_t)unit_part[r / rows] * rows + r % rows : r;
        const VT* xr = reinterpret_cast<const VT*>(X + src * d);
        // eight partial sums per lane (element c goes to sum (c / 64) % 8), added in order at the end
        VT q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) q[u] = (VT)(0.0f);
        int64_t base = 0;
        for (; base + 8 * 64 <= dv; base += 8 * 64) {  // wave-uniform
            VT x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(xr + base + u * 64 + lane);
#pragma unroll
            for (int u = 0; u < 8; ++u) q[u] += x[u] * tv[base + u * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t c = base + u * 64 + lane;
            if (c < dv) q[u] += xr[c] * tv[c];
        }
        const VT s = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        const float z = wave_sum(hsum(s));
        if (lane == 0) resid[r] = loss_slope<LOSS>(z, y[src]);
    }
}

template <bool VEC>
__global__ __launch_bounds__(256) void xtr_kernel(const float* __restrict__ X,
                                                  const float* __restrict__ resid,
                                                  float* __restrict__ partial, int64_t rows,
                                                  int64_t d, int chunks, int64_t rows_per_chunk,
                                                  const int* __restrict__ unit_part) {
    using VT = typename std::conditional<VEC, v4f, float>::type;
    const int64_t dv = VEC ? d / 4 : d;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y;
    const int j = blockIdx.z;  // unit
    if (c >= dv) return;
    const int64_t r0 = (int64_t)chunk * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const int part = unit_part ? unit_part[j] : j;
    const VT* xp = reinterpret_cast<const VT*>(X + ((int64_t)part * rows) * d) + c;
    const float* rp = resid + (int64_t)j * rows;
    VT acc = (VT)(0.0f);
    int64_t r = r0;
    for (; r + 8 <= r1; r += 8) {
        VT x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(xp + (r + u) * dv);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += rp[r + u] * x[u];
    }
    for (; r < r1; ++r) acc += rp[r] * xp[r * dv];
    reinterpret_cast<VT*>(partial)[((int64_t)j * chunks + chunk) * dv + c] = acc;
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
