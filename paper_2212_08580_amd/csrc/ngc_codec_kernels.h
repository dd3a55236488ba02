// Device code of the encode, decode and fused passes of libngc for gfx950 (CDNA4, wave64); the
// launchers are in ngc_codec.hip.  Every kernel here follows the canonical order of additions
// stated in ngc_dev_common.h.
#pragma once

#include <hip/hip_runtime.h>

#include "ngc_dev_common.h"

// ---------------------------------------------------------------------------
// A column tile of G in LDS: kp rows of 64 lanes' elements (row j at tile[j*64 + lane]);
// rows from k up to kp are zero so that four columns of B can always be taken at once.
// Staged by the block's WAVES waves, eight rows' loads in flight per wave.
// ---------------------------------------------------------------------------
template <typename VT, int WAVES>
__device__ __forceinline__ void stage_tile(VT* tile, const float* __restrict__ G, int k, int kp,
                                           int64_t d, int64_t c, bool in, int wave, int lane) {
    for (int r0 = wave; r0 < kp; r0 += 8 * WAVES) {
        VT v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + WAVES * u;
            v[u] = (VT)(0.0f);
            if (in && r < k) v[u] = *reinterpret_cast<const VT*>(G + (int64_t)r * d + c);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + WAVES * u;
            if (r < kp) tile[r * 64 + lane] = v[u];
        }
    }
}

// The same tile by way of registers, for a block of four waves and at most NGC_MAX_N rows: the
// loads of a whole tile are issued (sixteen per thread) and land in LDS later, so that they can
// be in flight while the block works on the tile that is in LDS now.
template <typename VT>
struct tile_regs {
    VT v[NGC_MAX_N / 4];
};

template <typename VT>
__device__ __forceinline__ void tile_fetch(tile_regs<VT>& t, const float* __restrict__ G, int k, int64_t d,
                                           int64_t c, bool in, int wave) {
#pragma unroll
    for (int u = 0; u < NGC_MAX_N / 4; ++u) {
        const int r = wave + 4 * u;
        t.v[u] = (VT)(0.0f);
        if (in && r < k) t.v[u] = __builtin_nontemporal_load(reinterpret_cast<const VT*>(G + (int64_t)r * d + c));  // read once: keep it out of the caches' way
    }
}

template <typename VT>
__device__ __forceinline__ void tile_land(VT* tile, const tile_regs<VT>& t, int kp, int wave, int lane) {
#pragma unroll
    for (int u = 0; u < NGC_MAX_N / 4; ++u) {
        const int r = wave + 4 * u;
        if (r < kp) tile[r * 64 + lane] = t.v[u];
    }
}

// Messages of the four workers of one group under one layer for this lane's columns:
//   m[r] = sum_j B[4g+r][j] * tile[j]   in ascending j, one fused multiply-add per term,
// on the matrix cores: v_mfma_f32_4x4x1_16B_f32 multiplies, in each of its sixteen blocks of
// four lanes, a column of four values (lane 4b+r holds coefficient r) by a row of four values
// (lane l holds its own tile element) and adds the 4 x 4 products to the accumulators, register
// r of lane l <- coefficient r times the element of lane l: one product per output and
// instruction, rounded once like a scalar fused multiply-add (checked bit for bit against fmaf,
// denormals included), four workers' terms per instruction at twice the vector pipe's rate.
// So lane l feeds coefficient l % 4 of the column, every lane gets all four messages, and the
// order of additions is the canonical one.
// cf holds the group's coefficients in trips of four columns, cf[jc*16 + r*4 + t] =
// B[4g+r][4jc+t]: one 16-byte load per lane and trip (component t = column 4jc+t).  Bit t of
// cmask says whether columns 4t..4t+3 touch the group's supports at all (a trip that does not
// is skipped).  The coefficients and tile rows of the next trip are requested before the
// multiply-adds of the current one are issued.
template <typename VT>
__device__ __forceinline__ void load_trip(const VT* tile, int lane, const float* __restrict__ cf, int jc,
                                          v4f& w, VT (&x)[4]) {
    w = *reinterpret_cast<const v4f*>(cf + jc * 16 + (lane & 3) * 4);
#pragma unroll
    for (int t = 0; t < 4; ++t) x[t] = tile[(4 * jc + t) * 64 + lane];
}

// acc[v]: the four messages' element v of this lane
template <typename VT, int V>
__device__ __forceinline__ void fma_trip(const v4f& w, const VT (&x)[4], v4f (&acc)[V]) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < V; ++v)
            acc[v] = __builtin_amdgcn_mfma_f32_4x4x1f32(w[t], ngc_get(x[t], v), acc[v], 0, 0, 0);
}

// Two register sets take the trips in turn, so the loads of the next trip are in flight during
// the multiply-adds of the current one without any copy between them.
template <typename VT, int V>
__device__ __forceinline__ void group_messages(const VT* tile, int lane, const float* __restrict__ cf,
                                               unsigned cmask, VT (&m)[4]) {
    v4f acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = (v4f)(0.0f);
    if (cmask != 0) {
        v4f wa, wb;
        VT xa[4], xb[4];
        load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wa, xa);
        cmask &= cmask - 1;
        for (;;) {
            if (cmask == 0) {
                fma_trip<VT, V>(wa, xa, acc);
                break;
            }
            load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wb, xb);
            cmask &= cmask - 1;
            fma_trip<VT, V>(wa, xa, acc);
            if (cmask == 0) {
                fma_trip<VT, V>(wb, xb, acc);
                break;
            }
            load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wa, xa);
            cmask &= cmask - 1;
            fma_trip<VT, V>(wb, xb, acc);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int v = 0; v < V; ++v) ngc_set(m[r], v, acc[v][r]);
}

// ---------------------------------------------------------------------------
// Encode.  Work items are (layer, group of four workers); they are dealt to the blocks of a
// column tile and to their waves in turn, layer index fastest, so that every wave gets rows
// of every layer (row weights differ by up to s_max + 1).  Message (u, i) is row u*n + i of
// C viewed as [L*n][d].
// ---------------------------------------------------------------------------
constexpr int ENC_WAVES = 8;

template <typename VT, int V>
__global__ __launch_bounds__(ENC_WAVES * 64) void encode_kernel(const float* __restrict__ G,
                                                                float* __restrict__ C,
                                                                const unsigned* __restrict__ gmask,
                                                                const float* __restrict__ gcoef, int n, int k,
                                                                int kp, int ng, int64_t d, int layer_begin,
                                                                int layer_count) {
    extern __shared__ float tile_raw[];
    VT* tile = reinterpret_cast<VT*>(tile_raw);  // [kp][64]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = ((int64_t)blockIdx.x * 64 + lane) * V;
    const bool in = c < d;
    stage_tile<VT, ENC_WAVES>(tile, G, k, kp, d, c, in, wave, lane);
    __syncthreads();
    const int items = layer_count * ng;
    const int stride = (int)gridDim.y * ENC_WAVES;
    for (int t = (int)blockIdx.y * ENC_WAVES + wave; t < items; t += stride) {
        const int u = layer_begin + t % layer_count;
        const int g = t / layer_count;
        const int ug = u * ng + g;
        VT m[4];
        group_messages<VT, V>(tile, lane, gcoef + (size_t)ug * kp * 4, gmask[ug], m);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * g + r;
            if (in && i < n) *reinterpret_cast<VT*>(C + ((int64_t)u * n + i) * d + c) = m[r];
        }
    }
}

// ---------------------------------------------------------------------------
// Decode.  g = sum_i a[i] * C[i][:] over the workers with a[i] != 0, in the canonical order:
// a block covers 16*V columns, its sixteen groups of 16 lanes hold the sixteen partial sums
// (worker i adds into number i mod 16), fp64 products and sums, one rounding.
// ---------------------------------------------------------------------------
struct decode_args {
    double a[NGC_MAX_N];  // zero at stragglers and beyond n
};

template <typename VT, int V>
__device__ __forceinline__ void decode_slot_sum(const float* __restrict__ Cl, int64_t d, int64_t c, bool in,
                                                int slot, const double* a, double (&acc)[V]) {
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
    if (!in) return;
    // a worker index has at most four candidates per partial sum (n <= 64): their loads go out together
    VT m[NGC_MAX_N / 16];
    double av[NGC_MAX_N / 16];
#pragma unroll
    for (int u = 0; u < NGC_MAX_N / 16; ++u) {
        const int i = slot + 16 * u;
        av[u] = a[i];
        m[u] = (VT)(0.0f);
        if (av[u] != 0.0) m[u] = *reinterpret_cast<const VT*>(Cl + (int64_t)i * d + c);
    }
#pragma unroll
    for (int u = 0; u < NGC_MAX_N / 16; ++u)
        if (av[u] != 0.0) {
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = __builtin_fma(av[u], (double)ngc_get(m[u], v), acc[v]);
        }
}

// thread q < 16*V adds the sixteen partial sums of column q of the block's tile in canonical order
template <int V>
__device__ __forceinline__ double combine16(const double* part, int pw, int q) {
    double w[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
        w[g] = ngc_quad(part[(4 * g) * pw + q], part[(4 * g + 1) * pw + q], part[(4 * g + 2) * pw + q],
                        part[(4 * g + 3) * pw + q]);
    return ngc_quad(w[0], w[1], w[2], w[3]);
}

template <typename VT, int V>
__global__ __launch_bounds__(256) void decode_kernel(const float* __restrict__ Cl, float* __restrict__ g,
                                                     int64_t d, decode_args args) {
    constexpr int PW = 16 * V + 1;
    __shared__ double part[16 * PW];
    const int lane16 = threadIdx.x & 15;
    const int slot = threadIdx.x >> 4;
    const int64_t c = ((int64_t)blockIdx.x * 16 + lane16) * V;
    double acc[V];
    decode_slot_sum<VT, V>(Cl, d, c, c < d, slot, args.a, acc);
#pragma unroll
    for (int v = 0; v < V; ++v) part[slot * PW + lane16 * V + v] = acc[v];
    __syncthreads();
    const int q = threadIdx.x;
    if (q < 16 * V) {
        const int64_t cq = (int64_t)blockIdx.x * 16 * V + q;
        if (cq < d) g[cq] = (float)combine16<V>(part, PW, q);
    }
}

// The same combination for long gradients (d of several hundred thousand): one thread per V
// columns, so a wave reads 64*V consecutive floats of a message at a time; the sixteen partial
// sums sit in registers, sixteen messages' loads are in flight together.
template <typename VT, int V>
__global__ __launch_bounds__(256) void decode_wide_kernel(const float* __restrict__ Cl,
                                                          float* __restrict__ g, int64_t d, int n,
                                                          decode_args args) {
    const int64_t c = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
    if (c >= d) return;
    double acc[16][V];
#pragma unroll
    for (int s = 0; s < 16; ++s)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[s][v] = 0.0;
    for (int base = 0; base < n; base += 16) {
        VT m[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            m[s] = (VT)(0.0f);
            if (args.a[base + s] != 0.0) m[s] = *reinterpret_cast<const VT*>(Cl + (int64_t)(base + s) * d + c);
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const double a = args.a[base + s];  // block-uniform
            if (a != 0.0) {
#pragma unroll
                for (int v = 0; v < V; ++v) acc[s][v] = __builtin_fma(a, (double)ngc_get(m[s], v), acc[s][v]);
            }
        }
    }
    VT out;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        double w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = ngc_quad(acc[4 * q][v], acc[4 * q + 1][v], acc[4 * q + 2][v], acc[4 * q + 3][v]);
        ngc_set(out, v, (float)ngc_quad(w[0], w[1], w[2], w[3]));
    }
    *reinterpret_cast<VT*>(g + c) = out;
}

// Decode with the decode vector taken from a row of the explicit decoding matrix A_sigma held
// on the device: the row is copied to LDS, then the combination runs as in decode_kernel.
template <typename VT, int V>
__global__ __launch_bounds__(256) void decode_lookup_kernel(const float* __restrict__ Cl,
                                                            float* __restrict__ g, int64_t d, int n,
                                                            const double* __restrict__ a_row) {
    constexpr int PW = 16 * V + 1;
    __shared__ double part[16 * PW];
    __shared__ double a_s[NGC_MAX_N];
    if (threadIdx.x < NGC_MAX_N) a_s[threadIdx.x] = (int)threadIdx.x < n ? a_row[threadIdx.x] : 0.0;
    __syncthreads();
    const int lane16 = threadIdx.x & 15;
    const int slot = threadIdx.x >> 4;
    const int64_t c = ((int64_t)blockIdx.x * 16 + lane16) * V;
    double acc[V];
    decode_slot_sum<VT, V>(Cl, d, c, c < d, slot, a_s, acc);
#pragma unroll
    for (int v = 0; v < V; ++v) part[slot * PW + lane16 * V + v] = acc[v];
    __syncthreads();
    const int q = threadIdx.x;
    if (q < 16 * V) {
        const int64_t cq = (int64_t)blockIdx.x * 16 * V + q;
        if (cq < d) g[cq] = (float)combine16<V>(part, PW, q);
    }
}

// ---------------------------------------------------------------------------
// Coded rounds: for each round r of a run of rounds, the messages of the round's layer
//   M[r][i][:] = fp32( sum_j B^(u_r)[i][j] G_r[j][:] )   for every worker with a_r[i] != 0
// and the recovered gradient  ghat[r][:] = fp32( sum_i a_r[i] * (double)M[r][i][:] ),
// from one tile of G in LDS: the tile is staged once per block when all rounds share G, once
// per round otherwise.  A block of four waves owns 64*V columns and a run of rounds.  Wave w
// takes the worker groups g = w, w+4, ...: worker 4g+r adds into partial sum 4w+r, which is
// partial sum (4g+r) mod 16 of the canonical decode order, so the sixteen partial sums of a
// column sit in the registers of four lanes (one per wave); each wave adds its four, the four
// results meet in LDS (two exchange areas used in turn, one barrier per round) and wave 0
// writes the round's gradient.  A message is rounded to fp32 and written before it is used.
// A round with layer < 0 (undecodable) writes a zero gradient and no message.
// ---------------------------------------------------------------------------
struct round_rec {
    double a[NGC_MAX_N];  // decode vector of the round, zero at stragglers and beyond n
    int layer;            // -1: undecodable
    int pad[15];
};
static_assert(sizeof(round_rec) == 576, "round record layout");

enum { ROUNDS_SINGLE = 0, ROUNDS_ONE_G = 1, ROUNDS_G_PER_ROUND = 2 };

template <typename VT, int V, int MODE>
__global__ __launch_bounds__(256) void coded_rounds_kernel(
    const float* __restrict__ G, int64_t g_stride, float* __restrict__ M, int64_t m_stride,
    float* __restrict__ ghat, const round_rec* __restrict__ recs, round_rec one,
    const unsigned* __restrict__ gmask, const float* __restrict__ gcoef, int n, int k, int kp, int ng,
    int64_t d, int ntiles, int rounds, int rounds_per_block) {
    extern __shared__ double lds_raw64[];
    double* xch = lds_raw64;                                   // [2][4][64*V]
    VT* tile = reinterpret_cast<VT*>(xch + 2 * 4 * 64 * V);    // [kp][64]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile_id = (int)(blockIdx.x % (unsigned)ntiles);
    const int chunk = (int)(blockIdx.x / (unsigned)ntiles);
    const int64_t c = ((int64_t)tile_id * 64 + lane) * V;
    const bool in = c < d;
    constexpr bool SINGLE = MODE == ROUNDS_SINGLE;
    const int r0 = chunk * rounds_per_block;
    const int r1 = rounds < r0 + rounds_per_block ? rounds : r0 + rounds_per_block;
    if (r0 >= r1) return;
    // With a G per round the next round's tile is fetched into registers before this round's
    // work starts and lands in LDS after it: its way from HBM is hidden behind the arithmetic.
    tile_regs<VT> next;
    if (MODE == ROUNDS_G_PER_ROUND) {
        tile_fetch<VT>(next, G + (int64_t)r0 * g_stride, k, d, c, in, wave);
        tile_land<VT>(tile, next, kp, wave, lane);
    } else {
        stage_tile<VT, 4>(tile, G, k, kp, d, c, in, wave, lane);
    }
    __syncthreads();
    // A round's record (layer, the decode weights of the wave's workers, the trip masks of its
    // groups) is wave-uniform and comes through scalar loads.  They are asked for a round ahead,
    // all at once: the layer and the sixteen weights at the start of the round before, the trip
    // masks (which need the layer) at its end, so that a group's work does not begin by waiting
    // for two loads in a row.  Wave w owns groups w, w+4, w+8, w+12 (GW = 4 at most).
    constexpr int GW = NGC_MAX_N / 16;
    auto load_rec = [&](int r, int& layer, double (&a)[GW][4]) {
        layer = SINGLE ? one.layer : recs[r].layer;
#pragma unroll
        for (int gi = 0; gi < GW; ++gi)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int i = 4 * (wave + 4 * gi) + rr;  // < NGC_MAX_N; the vector is zero beyond n
                a[gi][rr] = SINGLE ? one.a[i] : recs[r].a[i];
            }
    };
    auto load_masks = [&](int layer, unsigned (&gm)[GW]) {
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
            const int g = wave + 4 * gi;
            gm[gi] = (layer >= 0 && g < ng) ? gmask[layer * ng + g] : 0u;
        }
    };
    int layer, layer_n = -1;
    double aw[GW][4], aw_n[GW][4];
    unsigned gm[GW], gm_n[GW];
    load_rec(r0, layer, aw);
    load_masks(layer, gm);
    for (int r = r0; r < r1; ++r) {
        if (MODE == ROUNDS_G_PER_ROUND && r + 1 < r1)
            tile_fetch<VT>(next, G + (int64_t)(r + 1) * g_stride, k, d, c, in, wave);
        if (r + 1 < r1) load_rec(r + 1, layer_n, aw_n);
        double q[V];
#pragma unroll
        for (int v = 0; v < V; ++v) q[v] = 0.0;
        if (layer >= 0) {
            double acc[4][V];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int v = 0; v < V; ++v) acc[rr][v] = 0.0;
            float* Mr = M + (int64_t)r * m_stride + c;
#pragma unroll
            for (int gi = 0; gi < GW; ++gi) {
                const int g = wave + 4 * gi;
                const double(&av)[4] = aw[gi];
                const bool any = av[0] != 0.0 || av[1] != 0.0 || av[2] != 0.0 || av[3] != 0.0;
                if (g < ng && any) {  // wave-uniform; not taken for four stragglers in a row
                    VT m[4];
                    group_messages<VT, V>(tile, lane, gcoef + (size_t)(layer * ng + g) * kp * 4, gm[gi], m);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        if (av[rr] != 0.0) {  // wave-uniform
                            if (in)
                                __builtin_nontemporal_store(m[rr], reinterpret_cast<VT*>(Mr + (int64_t)(4 * g + rr) * d));
#pragma unroll
                            for (int v = 0; v < V; ++v)
                                acc[rr][v] = __builtin_fma(av[rr], (double)ngc_get(m[rr], v), acc[rr][v]);
                        }
                    }
                }
            }
#pragma unroll
            for (int v = 0; v < V; ++v) q[v] = ngc_quad(acc[0][v], acc[1][v], acc[2][v], acc[3][v]);
        }
        if (r + 1 < r1) load_masks(layer_n, gm_n);
        double* x = xch + (size_t)(r & 1) * 4 * 64 * V;
#pragma unroll
        for (int v = 0; v < V; ++v) x[(wave * V + v) * 64 + lane] = q[v];
        __syncthreads();
        if (wave == 0 && in) {
            VT out;
#pragma unroll
            for (int v = 0; v < V; ++v)
                ngc_set(out, v, (float)ngc_quad(x[(0 * V + v) * 64 + lane], x[(1 * V + v) * 64 + lane],
                                                x[(2 * V + v) * 64 + lane], x[(3 * V + v) * 64 + lane]));
            *reinterpret_cast<VT*>(ghat + (int64_t)r * d + c) = out;
        }
        if (MODE == ROUNDS_G_PER_ROUND && r + 1 < r1) {
            __syncthreads();  // every wave is done with this round's tile
            tile_land<VT>(tile, next, kp, wave, lane);
            __syncthreads();
        }
        layer = layer_n;
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
            gm[gi] = gm_n[gi];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) aw[gi][rr] = aw_n[gi][rr];
        }
    }
}

// ---------------------------------------------------------------------------
// Fused tail of one iteration for a tile of 16*V columns: sum of the gradient kernel's block
// partials (-> G), messages of every layer (-> C), decode with the given vector (-> g) and the
// descent update of theta, all from LDS, each step in the canonical order of the stand-alone
// kernels (same bits).  Threads: groups of 16 lanes; a lane owns V columns.  TAB_LDS: the
// compressed code tables are copied to LDS once per block; otherwise (tables too large for
// the LDS a block may have) they are read from global memory.
// ---------------------------------------------------------------------------
template <typename VT, int V, bool TAB_LDS>
__global__ __launch_bounds__(1024) void iteration_tail_kernel(
    const float* __restrict__ partial, int chunks, float* __restrict__ G, float* __restrict__ C,
    const int* __restrict__ rowptr, const int* __restrict__ col, const float* __restrict__ coef,
    int nnz, int n, int k, int L, int64_t d, int layer, decode_args args, float* __restrict__ g,
    float* __restrict__ theta, float scale) {
    extern __shared__ float lds_raw[];
    constexpr int PW = 16 * V + 1;
    double* part = reinterpret_cast<double*>(lds_raw);                 // [16][PW]
    VT* tile = reinterpret_cast<VT*>(part + 16 * PW);                  // [k][16]   G tile
    VT* msg = tile + (size_t)k * 16;                                   // [n][16]   messages of the decode layer
    int* rp_l = reinterpret_cast<int*>(msg + (size_t)n * 16);          // [L*n + 1]
    int* col_l = rp_l + L * n + 1;                                     // [nnz]
    float* coef_l = reinterpret_cast<float*>(col_l + nnz);             // [nnz]
    const int* rp_s = TAB_LDS ? rp_l : rowptr;
    const int* col_s = TAB_LDS ? col_l : col;
    const float* coef_s = TAB_LDS ? coef_l : coef;
    // blockDim.x / 16 groups of 16 lanes (16 to 64 of them) share out the partitions of step 1 and the
    // messages of step 2; the decode keeps to the first sixteen, one per partial sum
    const int lane16 = threadIdx.x & 15;
    const int slot = threadIdx.x >> 4;
    const int nslot = (int)blockDim.x >> 4;
    const int64_t c = ((int64_t)blockIdx.x * 16 + lane16) * V;
    const bool in = c < d;
    if (TAB_LDS) {
        for (int t = threadIdx.x; t <= L * n; t += (int)blockDim.x) rp_l[t] = rowptr[t];
        for (int t = threadIdx.x; t < nnz; t += (int)blockDim.x) {
            col_l[t] = col[t];
            coef_l[t] = coef[t];
        }
    }
    // 1. G tile = sum of block partials, chunks added in index order (sixteen loads in flight)
    for (int j = slot; j < k; j += nslot) {
        VT acc = (VT)(0.0f);
        if (in) {
            const float* p = partial + (int64_t)j * chunks * d + c;
            acc = *reinterpret_cast<const VT*>(p);
            int t = 1;
            for (; t + 16 <= chunks; t += 16) {
                VT x[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) x[u] = *reinterpret_cast<const VT*>(p + (int64_t)(t + u) * d);
#pragma unroll
                for (int u = 0; u < 16; ++u) acc += x[u];
            }
            if (t + 8 <= chunks) {
                VT x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const VT*>(p + (int64_t)(t + u) * d);
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += x[u];
                t += 8;
            }
            for (; t < chunks; ++t) acc += *reinterpret_cast<const VT*>(p + (int64_t)t * d);
            *reinterpret_cast<VT*>(G + (int64_t)j * d + c) = acc;
        }
        tile[j * 16 + lane16] = acc;
    }
    __syncthreads();
    // 2. messages of every (layer, worker) pair; those of the decode layer are kept in LDS
    const int np = L * n;
    for (int p = slot; p < np; p += nslot) {
        const int b = rp_s[p], e = rp_s[p + 1];
        VT m = (VT)(0.0f);
        int t = b;
        for (; t + 4 <= e; t += 4) {
            VT x[4];
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                w[u] = coef_s[t + u];
                x[u] = tile[col_s[t + u] * 16 + lane16];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) m = ngc_fma(w[u], x[u], m);
        }
        for (; t < e; ++t) m = ngc_fma(coef_s[t], tile[col_s[t] * 16 + lane16], m);
        if (in) *reinterpret_cast<VT*>(C + (int64_t)p * d + c) = m;
        if (p / n == layer) msg[(p - layer * n) * 16 + lane16] = m;
    }
    __syncthreads();
    // 3. decode: fp64 products and sums, worker i adds into partial sum i mod 16
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
    if (slot < 16) {
        for (int i = slot; i < n; i += 16) {
            const double a = args.a[i];
            if (a != 0.0) {
                const VT m = msg[i * 16 + lane16];
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] = __builtin_fma(a, (double)ngc_get(m, v), acc[v]);
            }
        }
#pragma unroll
        for (int v = 0; v < V; ++v) part[slot * PW + lane16 * V + v] = acc[v];
    }
    __syncthreads();
    const int q = threadIdx.x;
    if (q < 16 * V) {
        const int64_t cq = (int64_t)blockIdx.x * 16 * V + q;
        if (cq < d) {
            const float gq = (float)combine16<V>(part, PW, q);
            g[cq] = gq;
            // 4. theta <- theta - scale * g
            theta[cq] = theta[cq] - scale * gq;
        }
    }
}

// ---------------------------------------------------------------------------
// Worker-side encode: message of worker i under layer u formed from the partial gradients the
// worker computed itself, W[i][t] in task order,
//   C[u][i][:] = sum_t wcoef[u][i][t] * W[i][t][:]
// for every layer the worker has finished (unfinished ones are zero-filled).  By nesting, task
// t feeds every layer whose support contains its partition, so each W row is read once and
// added into the LMAX accumulators of the block's run of layers (blockIdx.z picks the run).
// Only the rows the worker has computed are read: at most sched_len[i], its own schedule.
// ---------------------------------------------------------------------------
struct worker_progress {
    unsigned char done[NGC_MAX_N];
};

template <typename VT, int V, int LMAX>
__global__ __launch_bounds__(64) void worker_encode_kernel(const float* __restrict__ W,
                                                           float* __restrict__ C,
                                                           const int* __restrict__ needed,
                                                           const int* __restrict__ sched_len,
                                                           const float* __restrict__ wcoef, int n,
                                                           int L, int T, int per_task, int64_t d,
                                                           worker_progress prog) {
    // T: rows of W per worker (partitions); prog.done counts atomic tasks of per_task partitions
    const int i = blockIdx.y;
    const int u0 = (int)blockIdx.z * LMAX;
    const int64_t c = ((int64_t)blockIdx.x * 64 + threadIdx.x) * V;
    if (c >= d) return;
    int done = prog.done[i] * per_task;
    done = done < sched_len[i] ? done : sched_len[i];
    VT acc[LMAX];
#pragma unroll
    for (int u = 0; u < LMAX; ++u) acc[u] = (VT)(0.0f);
    for (int t = 0; t < done; ++t) {
        const VT x = *reinterpret_cast<const VT*>(W + ((int64_t)i * T + t) * d + c);
#pragma unroll
        for (int u = 0; u < LMAX; ++u)
            if (u0 + u < L) acc[u] = ngc_fma(wcoef[((int64_t)(u0 + u) * n + i) * T + t], x, acc[u]);
    }
#pragma unroll
    for (int u = 0; u < LMAX; ++u)
        if (u0 + u < L) {
            const VT out = prog.done[i] >= needed[(u0 + u) * n + i] ? acc[u] : (VT)(0.0f);
            *reinterpret_cast<VT*>(C + ((int64_t)(u0 + u) * n + i) * d + c) = out;
        }
}
