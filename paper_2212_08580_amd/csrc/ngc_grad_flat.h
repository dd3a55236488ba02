// Partition gradients (least squares / logistic) for short rows (up to some 250 features) of
// any length: written for those whose length is no multiple of four.  Such rows are not 16-byte
// addressable one by one, but a run of them is one contiguous stretch of X, and that stretch
// is: the kernel reads it as it lies, in whole float4 from the 16-byte granule the run starts
// in, 1 KiB per wave and instruction, and sorts out rows afterwards.  The stretch of one trip
// goes through LDS unchanged; there (rows of fewer than 64 features) lane l picks up rows l,
// l+64, ... whole, one element per LDS read, so a row's margin x.theta and its update
// acc += r*x stay inside one lane and nothing crosses lanes until the block's final sum; longer
// rows are shared by four or eight lanes, see below.  (The lanes' reads are d words
// apart: no bank conflict for odd d; up to eight-way conflicts, d = 8 * odd, cost nothing
// measurable, the sixteen-way ones of d = 16 and 48 cost a third and d = 32 two thirds: 48 takes
// the padded layout below, 16 and 32 the kernels that load whole rows.)
// theta is wave-uniform then (scalar registers), the accumulators of a lane sit in registers, the
// next trip's float4 are in flight while this one is worked on.
//
// A block of four waves owns a run of rows of one partition and each wave a quarter of it
// (a quarter of the block partials that one-wave blocks would leave to be summed); the trips of
// a wave's run all start at the same offset (0..3 floats) inside their granule.  Loads
// never leave the run: vector indices are clamped to the last float4 of the trip and of the
// run (so no byte is fetched twice either), which is a whole float4 of X.  If X ends inside a
// granule (its float count is no multiple of four) the rows that reach into that granule (one
// row; up to three if d = 1) cannot be read that way; a block leaves them out of its trips and
// one lane per such row adds it at the end from single loads.
// Rows past the end of the run re-read the run's last row with weight 0.
// One partial per block, summed in block order by the reduction kernel.
#pragma once

#include <hip/hip_runtime.h>

#include "ngc_dev_common.h"
#include "ngc_grad_kernels.h"

// L lanes share a row (L = 1 for d < 64; 4 or 8 for longer rows): lane l works on row l / L of a
// pass and owns the h = ceil(d / L) columns from (l % L) * h on; the L partial margins meet
// through cross-lane exchanges in a fixed order.  DMAX: 2 or a multiple of 8, above h.
// A trip is R = 64 / DMAX passes of 64 / L rows.
// PAD (L = 1, d a multiple of 8): a row takes d + 4 words of LDS, its float4 land one slot
// further per row before them, and the lanes' reads are d + 4 words apart instead of d: for
// d = 48 that turns sixteen-way bank conflicts into four-way ones (5.3 -> 6.2 TB/s).
template <int DMAX, int L, int LOSS, bool PAD = false>
__global__ __launch_bounds__(256) void grad_flat_kernel(const float* __restrict__ X, const float* __restrict__ y,
                                                       const float* __restrict__ theta, float* __restrict__ partial,
                                                       int64_t rows, int chunks, int64_t rows_per_chunk,
                                                       const int* __restrict__ unit_part, int d, int64_t x_floats) {
    constexpr int R = 64 / DMAX;
    constexpr int PASS_ROWS = 64 / L;
    constexpr int TRIP_ROWS = PASS_ROWS * R;
    constexpr int NL = (R * DMAX + 3) / 4;  // float4 per lane that cover a trip wherever it starts (h < DMAX)
    static_assert(TRIP_ROWS % 4 == 0, "a trip is a whole number of float4");
    // an LDS read of column DMAX - 1 of the last part of a trip's last row stays inside the staging area
    static_assert(L == 1 || 64 * R > L + DMAX + 2, "staging area");
    static_assert(!PAD || (L == 1 && DMAX >= 16), "padded rows: d + 4 <= DMAX - 4, so a trip still fits");
    __shared__ v4f stage_all[4][NL * 64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    v4f* stage = stage_all[wave];
    float* flat = reinterpret_cast<float*>(stage);
    const int unit = blockIdx.x / chunks;
    const int j = unit_part ? unit_part[unit] : unit;
    const int c0 = blockIdx.x % chunks;
    // the block's run in four quarters, one per wave (rows_per_chunk is a multiple of 4)
    const int64_t quarter = rows_per_chunk >> 2;
    int64_t r0 = (int64_t)c0 * rows_per_chunk + wave * quarter;
    if (r0 > rows) r0 = rows;
    const int64_t r_end = rows < r0 + quarter ? rows : r0 + quarter;
    // rows r1 .. r_end - 1 of the run reach into the granule X ends in (at most three rows, and
    // only in the blocks at the very end of X)
    int64_t r1 = r_end;
    if (x_floats & 3) {
        const int64_t first = (x_floats & ~(int64_t)3) / d - (int64_t)j * rows;  // first such row of this partition
        if (first < r1) r1 = first > r0 ? first : r0;
    }
    const float* yp = y + (int64_t)j * rows;
    const int64_t f0 = ((int64_t)j * rows + r0) * d;  // first float of the run
    const int shift = (int)(f0 & 3);
    const v4f* xv = reinterpret_cast<const v4f*>(X) + (f0 >> 2);
    const int trip_vecs = (TRIP_ROWS / 4) * d;
    const int trip_last = trip_vecs - (shift == 0);       // last float4 of a trip, counted from its first
    const int nl = trip_last / 64 + 1;                    // <= NL
    // last float4 the run needs, counted from its first: the one that holds the last float of
    // row r1 - 1, a whole float4 of X.  Lanes past the end of a trip or of the run re-read those.
    const int64_t run_last = ((((int64_t)j * rows + r1) * d - 1) >> 2) - (f0 >> 2);
    // this lane's row within a pass and its columns cbase .. cbase + hc - 1
    const int prow = lane / L;
    const int h = (d + L - 1) / L;
    const int cbase = (lane % L) * h;
    const int hc = d - cbase < h ? (d - cbase > 0 ? d - cbase : 0) : h;
    float th[DMAX], acc[DMAX];
#pragma unroll
    for (int c = 0; c < DMAX; ++c) {
        th[c] = c < hc ? theta[cbase + c] : 0.0f;
        acc[c] = 0.0f;
    }
    const int64_t ntrips = r0 < r1 ? (r1 - r0 + TRIP_ROWS - 1) / TRIP_ROWS : 0;
    if (ntrips > 0) {
        const int64_t last = r1 - 1;
        v4f s[NL];
        float yn[R];
        // LDS slot of this lane's u-th float4 of a trip (the same in every trip)
        int slot[NL];
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int v = u * 64 + lane;
            slot[u] = PAD ? v + v / (d >> 2) : v;
        }
        const int pitch = PAD ? d + 4 : d;
        auto fetch = [&](int64_t t) {
            // wave-uniform base and room, a 32-bit offset per lane
            int64_t vb = t * trip_vecs;
            vb = vb < run_last ? vb : run_last;
            const int64_t room64 = run_last - vb;
            const int room = room64 < trip_last ? (int)room64 : trip_last;
            const v4f* tb = xv + vb;
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                if (u < nl) {  // wave-uniform
                    const int rel = u * 64 + lane;
                    s[u] = __builtin_nontemporal_load(tb + (rel < room ? rel : room));
                }
            }
#pragma unroll
            for (int i = 0; i < R; ++i) {
                int64_t r = r0 + t * TRIP_ROWS + prow + PASS_ROWS * i;
                r = r < last ? r : last;
                yn[i] = yp[r];
            }
        };
        fetch(0);
        for (int64_t t = 0; t < ntrips; ++t) {
#pragma unroll
            for (int u = 0; u < NL; ++u)
                if (u < nl) stage[slot[u]] = s[u];
            float yc[R];
#pragma unroll
            for (int i = 0; i < R; ++i) yc[i] = yn[i];
            fetch(t + 1);  // past the run's end: clamped re-reads, never used
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int64_t left = r1 - (r0 + t * TRIP_ROWS);  // live rows from this trip's start on, >= 1
            const int lim = (int)(left < TRIP_ROWS ? left : TRIP_ROWS) - 1;
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int rit = prow + PASS_ROWS * i;
                const int rr = rit < lim ? rit : lim;
                const float* xr = flat + shift + rr * pitch + cbase;
                float x[DMAX];
#pragma unroll
                for (int c = 0; c < DMAX; ++c) x[c] = c < hc ? xr[c] : 0.0f;
                float z = 0.0f;
#pragma unroll
                for (int c = 0; c < DMAX; ++c) z = __builtin_fmaf(x[c], th[c], z);
#pragma unroll
                for (int m = 1; m < L; m <<= 1) z += __shfl_xor(z, m, 64);
                const float res = loss_slope<LOSS>(z, yc[i]) * (rit <= lim ? 1.0f : 0.0f);
#pragma unroll
                for (int c = 0; c < DMAX; ++c) acc[c] = __builtin_fmaf(res, x[c], acc[c]);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (prow < r_end - r1) {
        const int64_t r = r1 + prow;
        const float* xr = X + ((int64_t)j * rows + r) * d;
        float z = 0.0f;
        for (int c = 0; c < d; ++c) z = __builtin_fmaf(xr[c], theta[c], z);
        const float res = loss_slope<LOSS>(z, yp[r]);
#pragma unroll
        for (int c = 0; c < DMAX; ++c)
            if (c < hc) acc[c] = __builtin_fmaf(res, xr[cbase + c], acc[c]);
    }
    // block sum: a column's accumulators (one per wave and row of a pass), added in wave and
    // lane order by one thread per column (stride 65 words: h * 65 floats fit a wave's staging
    // area, and the readers' banks differ)
    static_assert((DMAX - 1) * 65 <= NL * 64 * 4, "block sum area");
#pragma unroll
    for (int c = 0; c < DMAX; ++c)
        if (c < h) flat[c * 65 + lane] = acc[c];
    __syncthreads();
    if ((int)threadIdx.x < d) {
        const int part = threadIdx.x / h, c = threadIdx.x - part * h;
        float sum = 0.0f;
        for (int w = 0; w < 4; ++w) {
            const float* fw = reinterpret_cast<const float*>(stage_all[w]) + c * 65 + part;
            for (int g = 0; g < PASS_ROWS; ++g) sum += fw[g * L];
        }
        partial[(int64_t)blockIdx.x * d + threadIdx.x] = sum;
    }
}

// G[j][:] = sum over chunks of partial[j][chunk][:], chunks added in index order, for launches
// that leave many block partials per partition (short rows: hundreds to a thousand): the same
// sum, term by term, as reduce_partials_kernel, with sixteen loads of a thread in flight instead
// of four (a thread's additions wait for memory, not for each other).
template <typename VT>
__global__ __launch_bounds__(64) void reduce_partials_deep_kernel(const VT* __restrict__ partial, VT* __restrict__ G,
                                                                  int64_t dv, int chunks,
                                                                  const int* __restrict__ unit_row) {
    const int64_t c = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y;
    if (c >= dv) return;
    const VT* p = partial + (int64_t)j * chunks * dv + c;
    VT acc = p[0];
    int t = 1;
    for (; t + 16 <= chunks; t += 16) {
        VT a[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) a[u] = p[(int64_t)(t + u) * dv];
#pragma unroll
        for (int u = 0; u < 16; ++u) acc += a[u];
    }
    for (; t < chunks; ++t) acc += p[(int64_t)t * dv];
    G[(int64_t)(unit_row ? unit_row[j] : j) * dv + c] = acc;
}
