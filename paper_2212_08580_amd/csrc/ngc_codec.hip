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
#include <cstring>
#include <thread>
#include <vector>

#include "ngc_dev_common.h"

// ---------------------------------------------------------------------------
// Code tables on the device.  Layout of d_code:
//   int   rowptr[L*n + 1] | int col[nnz] | float coef[nnz]      compressed rows, all layers
//   u32   gmask[L*ng]                (64-byte aligned)  bit t: one of the columns 4t..4t+3 is in the
//                                                       support of one of the workers 4g..4g+3
//   float gcoef[L*ng][kp][4]         (64-byte aligned)  gcoef[(u*ng+g)*kp + j][r] = B^(u)[4g+r][j]
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
                gcoef[(((size_t)u * ng + g) * kp + lc.col[t]) * 4 + r] = (float)lc.coef[t];
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
        if (in && r < k) t.v[u] = *reinterpret_cast<const VT*>(G + (int64_t)r * d + c);
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
//   m[r] = sum_j cf[j][r] * tile[j]   in ascending j, one fused multiply-add per term.
// cf and cmask are wave-uniform (scalar loads); four columns of B are taken per trip, bit t of
// cmask says whether columns 4t..4t+3 touch the group's supports at all (a trip that does not
// is skipped).  The coefficients and tile rows of the next trip are requested before the
// multiply-adds of the current one are issued.
template <typename VT>
__device__ __forceinline__ void load_trip(const VT* tile, int lane, const float* __restrict__ cf, int jc,
                                          float (&w)[16], VT (&x)[4]) {
#pragma unroll
    for (int t = 0; t < 16; ++t) w[t] = cf[jc * 16 + t];
#pragma unroll
    for (int t = 0; t < 4; ++t) x[t] = tile[(4 * jc + t) * 64 + lane];
}

// ROWS: bit r set = message r of the group is wanted (a straggler's message is not formed)
template <typename VT, int ROWS>
__device__ __forceinline__ void fma_trip(const float (&w)[16], const VT (&x)[4], VT (&m)[4]) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((ROWS >> r) & 1) m[r] = ngc_fma(w[t * 4 + r], x[t], m[r]);
}

// Two register sets take the trips in turn, so the loads of the next trip are in flight during
// the multiply-adds of the current one without any copy between them.
template <typename VT, int ROWS>
__device__ __forceinline__ void group_messages(const VT* tile, int lane, const float* __restrict__ cf,
                                               unsigned cmask, VT (&m)[4]) {
#pragma unroll
    for (int r = 0; r < 4; ++r) m[r] = (VT)(0.0f);
    if (cmask == 0) return;
    float wa[16], wb[16];
    VT xa[4], xb[4];
    load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wa, xa);
    cmask &= cmask - 1;
    for (;;) {
        if (cmask == 0) {
            fma_trip<VT, ROWS>(wa, xa, m);
            break;
        }
        load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wb, xb);
        cmask &= cmask - 1;
        fma_trip<VT, ROWS>(wa, xa, m);
        if (cmask == 0) {
            fma_trip<VT, ROWS>(wb, xb, m);
            break;
        }
        load_trip<VT>(tile, lane, cf, __builtin_ctz(cmask), wa, xa);
        cmask &= cmask - 1;
        fma_trip<VT, ROWS>(wb, xb, m);
    }
}

// The same with the wanted rows known only at run time (wave-uniform): one of sixteen variants.
template <typename VT>
__device__ __forceinline__ void group_messages_rows(const VT* tile, int lane, const float* __restrict__ cf,
                                                    unsigned cmask, int rows, VT (&m)[4]) {
    switch (rows) {
#define NGC_ROWS_CASE(R) case R: group_messages<VT, R>(tile, lane, cf, cmask, m); break;
        NGC_ROWS_CASE(1) NGC_ROWS_CASE(2) NGC_ROWS_CASE(3) NGC_ROWS_CASE(4) NGC_ROWS_CASE(5)
        NGC_ROWS_CASE(6) NGC_ROWS_CASE(7) NGC_ROWS_CASE(8) NGC_ROWS_CASE(9) NGC_ROWS_CASE(10)
        NGC_ROWS_CASE(11) NGC_ROWS_CASE(12) NGC_ROWS_CASE(13) NGC_ROWS_CASE(14) NGC_ROWS_CASE(15)
#undef NGC_ROWS_CASE
        default: break;
    }
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
        group_messages<VT, 15>(tile, lane, gcoef + (size_t)ug * kp * 4, gmask[ug], m);
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
    for (int r = r0; r < r1; ++r) {
        if (MODE == ROUNDS_G_PER_ROUND && r + 1 < r1)
            tile_fetch<VT>(next, G + (int64_t)(r + 1) * g_stride, k, d, c, in, wave);
        const int layer = SINGLE ? one.layer : recs[r].layer;
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
            for (int g = wave; g < ng; g += 4) {
                const int ug = layer * ng + g;
                double av[4];
                int rows = 0;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    av[rr] = SINGLE ? one.a[4 * g + rr] : recs[r].a[4 * g + rr];  // index < NGC_MAX_N; zero beyond n
                    rows |= (av[rr] != 0.0) << rr;
                }
                if (rows == 0) continue;  // wave-uniform: four stragglers in a row
                VT m[4];
                group_messages_rows<VT>(tile, lane, gcoef + (size_t)ug * kp * 4, gmask[ug], rows, m);
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
#pragma unroll
            for (int v = 0; v < V; ++v) q[v] = ngc_quad(acc[0][v], acc[1][v], acc[2][v], acc[3][v]);
        }
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
    }
}

// ---------------------------------------------------------------------------
// Fused tail of one iteration for a tile of 16*V columns: sum of the gradient kernel's block
// partials (-> G), messages of every layer (-> C), decode with the given vector (-> g) and the
// descent update of theta, all from LDS, each step in the canonical order of the stand-alone
// kernels (same bits).  Threads: 16 groups of 16 lanes; a lane owns V columns.  TAB_LDS: the
// compressed code tables are copied to LDS once per block; otherwise (tables too large for
// the LDS a block may have) they are read from global memory.
// ---------------------------------------------------------------------------
template <typename VT, int V, bool TAB_LDS>
__global__ __launch_bounds__(256) void iteration_tail_kernel(
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
    const int lane16 = threadIdx.x & 15;
    const int slot = threadIdx.x >> 4;
    const int64_t c = ((int64_t)blockIdx.x * 16 + lane16) * V;
    const bool in = c < d;
    if (TAB_LDS) {
        for (int t = threadIdx.x; t <= L * n; t += 256) rp_l[t] = rowptr[t];
        for (int t = threadIdx.x; t < nnz; t += 256) {
            col_l[t] = col[t];
            coef_l[t] = coef[t];
        }
    }
    // 1. G tile = sum of block partials, chunks added in index order (sixteen loads in flight)
    for (int j = slot; j < k; j += 16) {
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
    for (int p = slot; p < np; p += 16) {
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
    // runs of rounds per block: about eight blocks per CU in all, so that the tail of the launch is short
    int64_t chunks = std::max<int64_t>(1, std::min<int64_t>(rounds, (8 * (int64_t)ctx->cu_count + ntiles - 1) / ntiles));
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
    if (count <= ctx->rounds_cap) return NGC_OK;
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
    // a solve costs about n^2 / 1500 microseconds; a thread is worth starting per quarter of a
    // millisecond of such work (starting and joining one costs tens of microseconds, far more on a
    // host whose cores are busy), so small jobs stay on the calling thread
    const unsigned hw = std::max(1u, std::thread::hardware_concurrency());
    const double work_us = (double)rounds * ctx->n * ctx->n / 1500.0;
    const int nthreads = (int)std::min<double>(std::min(hw, 16u), std::max(1.0, work_us / 250.0));
    if (nthreads <= 1) {
        plan(0, rounds);
    } else {
        std::vector<std::thread> pool;
        const int per = (rounds + nthreads - 1) / nthreads;
        for (int t = 1; t < nthreads; ++t) pool.emplace_back(plan, std::min(rounds, t * per), std::min(rounds, (t + 1) * per));
        plan(0, std::min(rounds, per));
        for (auto& th : pool) th.join();
    }
    for (int r = 0; r < rounds; ++r) {
        if (status[r] != NGC_OK)
            return ngc_fail(ctx, status[r], status[r] == NGC_ERR_STATE ? "a chosen layer has no code yet"
                                                                       : "decode residual above tolerance in round " + std::to_string(r));
        if (layers_out) layers_out[r] = recs[r].layer;
        if (a_out) std::memcpy(a_out + (size_t)r * n, recs[r].a, sizeof(double) * n);
    }
    NGC_HIP(ctx, hipMemcpyAsync(ctx->d_rounds, recs, sizeof(round_rec) * (size_t)rounds, hipMemcpyHostToDevice, ctx->stream));
    NGC_HIP(ctx, hipEventRecord(ctx->rounds_ev, ctx->stream));
    ctx->rounds_ev_set = true;
    round_rec none;
    std::memset(&none, 0, sizeof(none));
    if (g_round_stride != 0)
        return launch_rounds<ROUNDS_G_PER_ROUND>(ctx, G_dev, g_round_stride, M_dev, m_round_stride, g_dev,
                                                 (const round_rec*)ctx->d_rounds, none, rounds);
    return launch_rounds<ROUNDS_ONE_G>(ctx, G_dev, 0, M_dev, m_round_stride, g_dev,
                                       (const round_rec*)ctx->d_rounds, none, rounds);
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
    ngc_prof_scope ps(ctx, NGC_KERNEL_TAIL);
#define NGC_TAIL_ARGS partial, chunks, G_dev, C_dev, cv.rowptr, cv.col, cv.coef, cv.nnz, n, k, L, d, layer, args, g_dev, theta_dev, (float)scale
#define NGC_TAIL_LAUNCH(VT, VV)                                                                                          \
    do {                                                                                                                 \
        if (tables)                                                                                                      \
            hipLaunchKernelGGL((iteration_tail_kernel<VT, VV, true>), dim3((unsigned)gx), dim3(256), lds, ctx->stream, NGC_TAIL_ARGS); \
        else                                                                                                             \
            hipLaunchKernelGGL((iteration_tail_kernel<VT, VV, false>), dim3((unsigned)gx), dim3(256), lds, ctx->stream, NGC_TAIL_ARGS); \
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
