// Partition gradients of the 2-layer perceptron (softmax cross-entropy of
// relu(x W1 + b1) W2 + b2), the third loss of ngc_partition_grads: the partial
// gradient g_j of Sec. II-C for each row block j, a plain sum over its rows.
//
// Device steps, all partitions at once:
//   1. H = relu(X W1 + b1)                 fp32 MFMA GEMM, bias + ReLU in the epilogue
//   2. per row: Z2 = H W2 + b2, P = softmax(Z2), dZ2 = P - onehot(label);
//      then dW2 += H^T dZ2, db2 += dZ2; dZ1 = (dZ2 W2^T) * [H > 0] written over H;
//      db1 += dZ1 (block partials).  One pass over H for a hidden layer of 1024 units
//      (mlp_head1024_kernel), else a pass that reads H and one that reads and writes it
//   3. dW1_j = X_j^T dZ1_j                 fp32 MFMA GEMM per partition, written into G
//   4. fixed-order sums: the block partials of step 2 into the tail of G, and the pieces of
//      the tiles of step 3 that were cut along K
//
// MFMA tile: v_mfma_f32_32x32x2_f32.  A block of 4 waves computes a 128 x 128
// tile of the output, each wave 64 x 64 as 2 x 2 MFMA blocks; operand tiles are
// staged in LDS k-major ([k][m] and [k][n]) so that the 32 lanes that feed one
// MFMA column read consecutive words.  Within a wave, MFMA block bm holds the
// tile rows 2*i + bm (i = MFMA row), so a lane fetches its two A values (and two
// B values) with one 8-byte LDS read and stores two adjacent output columns.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "ngc_internal.h"

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

#define NGC_HIP(ctx, call)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return ngc_fail(ctx, NGC_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

namespace {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDT = BM + 4;  // LDS row stride in floats (BM == BN)

enum { EPI_STORE = 0, EPI_BIAS_RELU = 1 };

// 4 consecutive elements starting at p[0], of which `left` are inside the matrix
__device__ __forceinline__ v4f load4(const float* __restrict__ p, int64_t left, bool vec_ok) {
    v4f v = (v4f)(0.0f);
    if (left >= 4 && vec_ok) {
        v = *reinterpret_cast<const v4f*>(p);
    } else {
        if (left > 0) v.x = p[0];
        if (left > 1) v.y = p[1];
        if (left > 2) v.z = p[2];
        if (left > 3) v.w = p[3];
    }
    return v;
}

// Blocks are handed to the 8 XCDs in turn (block b runs on XCD b % 8) and each XCD
// has its own L2.  This renumbering gives every XCD one contiguous run of tiles in
// column-tile-fastest order, so that the tiles sharing a row panel of A (and the
// panels of one batch entry) meet in the same L2 instead of being fetched by all
// eight.
struct tile_id {
    int x, y, z;
};
__device__ __forceinline__ tile_id xcd_tile() {
    const int gx = gridDim.x, gy = gridDim.y, gz = gridDim.z;
    const int total = gx * gy * gz;
    const int b = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
    const int per = total / 8;
    const int v = b < per * 8 ? (b % 8) * per + b / 8 : b;
    tile_id t;
    t.x = v % gx;
    t.y = (v / gx) % gy;
    t.z = v / (gx * gy);
    return t;
}

// C[M x N] = A * B (+ epilogue), batched over blockIdx.z.
//   A_KMAJOR: A is stored [K][M] (element (m,k) at A[k*lda + m]); else [M][K].
//   B is stored [K][N].  C is stored [M][N].
//   Batch entry z reads A at batch index a_batch[z] and writes C at c_batch[z]
//   (z itself where the map is null): several entries may read the same A.
template <bool A_KMAJOR, int EPI>
__global__ __launch_bounds__(256, 2) void mlp_gemm_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C,
    const float* __restrict__ bias, int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
    int64_t strideA, int64_t strideB, int64_t strideC, int a_vec_ok, int b_vec_ok, int c_vec_ok,
    const int* __restrict__ a_batch, const int* __restrict__ c_batch) {
    __shared__ float As[2][BK][LDT];
    __shared__ float Bs[2][BK][LDT];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const tile_id tile = xcd_tile();
    const int m0 = tile.y * BM, n0 = tile.x * BN;
    A += (int64_t)(a_batch ? a_batch[tile.z] : tile.z) * strideA;
    B += (int64_t)tile.z * strideB;
    C += (int64_t)(c_batch ? c_batch[tile.z] : tile.z) * strideC;

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Tiles that lie wholly inside the matrices and are 16-byte addressable, with K a
    // whole number of k tiles, take the fast loads: one unguarded vector load per
    // operand piece and nothing else, so that the main loop below has no branch
    // and the compiler can count the loads in flight (a wait before a stage's LDS
    // stores then covers that stage only; with a branch around any load it has to
    // wait for every outstanding load, the ones just issued included).  Edge
    // tiles and odd leading dimensions take the guarded element-wise loads.
    const bool a_inside = a_vec_ok && (m0 + BM <= M);
    const bool b_inside = b_vec_ok && (n0 + BN <= N);
    const bool fast = a_inside && b_inside && (K % BK == 0);
    auto gload_fast = [&](int k0, v4f (&ra)[2], v4f (&rb)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int idx = t + h * 256;
            if (A_KMAJOR) {
                const int k = idx >> 5, m4 = (idx & 31) * 4;
                ra[h] = *reinterpret_cast<const v4f*>(A + (int64_t)(k0 + k) * lda + m0 + m4);
            } else {
                const int m = idx >> 2, k4 = (idx & 3) * 4;
                ra[h] = *reinterpret_cast<const v4f*>(A + (int64_t)(m0 + m) * lda + k0 + k4);
            }
            const int k = idx >> 5, n4 = (idx & 31) * 4;
            rb[h] = *reinterpret_cast<const v4f*>(B + (int64_t)(k0 + k) * ldb + n0 + n4);
        }
    };
    auto gload = [&](int k0, v4f (&ra)[2], v4f (&rb)[2]) {
        const bool k_inside = k0 + BK <= K;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int idx = t + h * 256;
            if (A_KMAJOR) {
                const int k = idx >> 5, m4 = (idx & 31) * 4;
                const int gk = k0 + k, gm = m0 + m4;
                const float* p = A + (int64_t)gk * lda + gm;
                if (a_inside && k_inside)
                    ra[h] = *reinterpret_cast<const v4f*>(p);
                else
                    ra[h] = (gk < K) ? load4(p, (int64_t)M - gm, a_vec_ok) : (v4f)(0.0f);
            } else {
                const int m = idx >> 2, k4 = (idx & 3) * 4;
                const int gm = m0 + m, gk = k0 + k4;
                const float* p = A + (int64_t)gm * lda + gk;
                if (a_inside && k_inside)
                    ra[h] = *reinterpret_cast<const v4f*>(p);
                else
                    ra[h] = (gm < M) ? load4(p, (int64_t)K - gk, a_vec_ok) : (v4f)(0.0f);
            }
            const int k = idx >> 5, n4 = (idx & 31) * 4;
            const int gk = k0 + k, gn = n0 + n4;
            const float* q = B + (int64_t)gk * ldb + gn;
            if (b_inside && k_inside)
                rb[h] = *reinterpret_cast<const v4f*>(q);
            else
                rb[h] = (gk < K) ? load4(q, (int64_t)N - gn, b_vec_ok) : (v4f)(0.0f);
        }
    };
    auto sstore = [&](int buf, const v4f (&ra)[2], const v4f (&rb)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int idx = t + h * 256;
            if (A_KMAJOR) {
                const int k = idx >> 5, m4 = (idx & 31) * 4;
                *reinterpret_cast<v4f*>(&As[buf][k][m4]) = ra[h];
            } else {
                const int m = idx >> 2, k4 = (idx & 3) * 4;
                As[buf][k4 + 0][m] = ra[h].x;
                As[buf][k4 + 1][m] = ra[h].y;
                As[buf][k4 + 2][m] = ra[h].z;
                As[buf][k4 + 3][m] = ra[h].w;
            }
            const int k = idx >> 5, n4 = (idx & 31) * 4;
            *reinterpret_cast<v4f*>(&Bs[buf][k][n4]) = rb[h];
        }
    };

    auto compute = [&](int buf) {
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            const int k = 2 * kk + lhi;
            const v2f a2 = *reinterpret_cast<const v2f*>(&As[buf][k][wm * 64 + 2 * l32]);
            const v2f b2 = *reinterpret_cast<const v2f*>(&Bs[buf][k][wn * 64 + 2 * l32]);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, b2.x, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, b2.y, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, b2.x, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, b2.y, acc[1][1], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // Software pipeline, two k tiles deep: while tile kt is multiplied out of LDS,
    // tile kt+1 waits in registers for its turn in the other LDS buffer and tile
    // kt+2 is on its way from memory.  Two register stages (p, q) alternate, the
    // loop is unrolled twice so that each has a fixed role.  Fast tiles run the
    // pairs that need no end-of-K test in a loop without conditions; the guarded
    // loop finishes (or, for the other tiles, does) the rest.
    const int nk = (K + BK - 1) / BK;
    v4f pa[2], pb[2], qa[2], qb[2];
    int kt = 0;
    if (fast) {
        gload_fast(0, pa, pb);
        sstore(0, pa, pb);
        if (nk > 1) gload_fast(BK, qa, qb);
        __syncthreads();
        // the scheduling barriers keep the loads where they are written, ahead of the
        // multiplication (left alone, the scheduler moves them down towards their use)
        for (; kt + 3 < nk; kt += 2) {
            gload_fast((kt + 2) * BK, pa, pb);
            __builtin_amdgcn_sched_barrier(0);
            compute(0);
            __builtin_amdgcn_sched_barrier(0);
            sstore(1, qa, qb);
            __syncthreads();
            gload_fast((kt + 3) * BK, qa, qb);
            __builtin_amdgcn_sched_barrier(0);
            compute(1);
            __builtin_amdgcn_sched_barrier(0);
            sstore(0, pa, pb);
            __syncthreads();
        }
    } else {
        gload(0, pa, pb);
        sstore(0, pa, pb);
        if (nk > 1) gload(BK, qa, qb);
        __syncthreads();
    }
    for (; kt < nk; kt += 2) {
        // even tile kt from buffer 0; q holds tile kt+1
        if (kt + 2 < nk) gload((kt + 2) * BK, pa, pb);
        compute(0);
        if (kt + 1 < nk) sstore(1, qa, qb);
        __syncthreads();
        // odd tile kt+1 from buffer 1; p holds tile kt+2
        if (kt + 3 < nk) gload((kt + 3) * BK, qa, qb);
        if (kt + 1 < nk) compute(1);
        if (kt + 2 < nk) sstore(0, pa, pb);
        __syncthreads();
    }

    // MFMA 32x32 result layout: register r of lane l is element (row, col) with
    // col = l % 32 and row = (r / 4) * 8 + (l / 32) * 4 + r % 4.
    const int gn = n0 + wn * 64 + 2 * l32;
    float bias0 = 0.0f, bias1 = 0.0f;
    if (EPI == EPI_BIAS_RELU) {
        if (gn < N) bias0 = bias[gn];
        if (gn + 1 < N) bias1 = bias[gn + 1];
    }
#pragma unroll
    for (int bm = 0; bm < 2; ++bm) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = (r >> 2) * 8 + lhi * 4 + (r & 3);
            const int gm = m0 + wm * 64 + 2 * i + bm;
            if (gm >= M) continue;
            float v0 = acc[bm][0][r], v1 = acc[bm][1][r];
            if (EPI == EPI_BIAS_RELU) {
                v0 = fmaxf(v0 + bias0, 0.0f);
                v1 = fmaxf(v1 + bias1, 0.0f);
            }
            float* out = C + (int64_t)gm * ldc + gn;
            if (gn + 1 < N && c_vec_ok) {
                v2f v;
                v.x = v0;
                v.y = v1;
                *reinterpret_cast<v2f*>(out) = v;
            } else {
                if (gn < N) out[0] = v0;
                if (gn + 1 < N) out[1] = v1;
            }
        }
    }
}

// Variant for outputs whose row count suits tiles of 112 better than tiles of 128
// (784 = 7 * 112): C[M x N] = A^T-stored-k-major * B, A at A[k*lda + m], batched
// over blockIdx.z.  v_mfma_f32_16x16x4_f32; a block of 4 waves computes a
// 112 x 128 tile, wave w the 112 x 32 slab of columns 32w.., as 7 x 2 MFMA blocks.
// Lane l feeds element (row or column l % 16, depth l / 16) of each operand block
// and holds rows 4*(l/16)..+3 of column l % 16 of each result block.
// LDS row strides: the four 16-lane groups of a wave read 16 consecutive words of four
// consecutive k rows, so a stride of 16 or 48 modulo 64 words puts the four groups on four
// disjoint sets of 16 banks (112 = 64 + 48 needs no padding, 128 gets 16 words).
constexpr int TM = 112, TN = 128, TK = 8, LDA = TM, LDB = TN + 16;
typedef float v4acc __attribute__((ext_vector_type(4)));

// How a launch whose tile count is no multiple of the CU count is evened out (FAST only).
// The tiles of one XCD's run (`per` of them, see xcd_tile) are `whole` tiles that are
// computed as they are, a multiple of the XCD's CU count, and per - whole tiles that are cut
// along K into `pieces` pieces each; a piece goes to a scratch tile and a second kernel adds
// the pieces of a tile in piece order.  The launch is one-dimensional: block b works for XCD
// b % 8 and is its item b / 8, whole tiles first, so the short items fill the gaps at the end.
// pieces == 0: the plain three-dimensional launch, one block per tile.
struct k_split {
    int pieces, per, whole, gx, gy;
    float* scratch;  // [8 * (per - whole) * pieces][TM][TN]
};

// 8-deep k tiles and one float4 of each operand per thread and stage keep the kernel
// under 100 registers and 16 KiB of LDS, so five blocks fit a CU: 1280 slots for the
// 1120 tiles of the 20 x 784 x 1024 backward product, which then run as one resident set
// instead of a full round plus a mostly empty one.
template <bool FAST>
__global__ __launch_bounds__(256, 5) void mlp_gemm112_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C, int M, int N,
    int K, int64_t lda, int64_t ldb, int64_t ldc, int64_t strideA, int64_t strideB,
    int64_t strideC, int a_vec_ok, int b_vec_ok, const int* __restrict__ a_batch,
    const int* __restrict__ c_batch, const k_split split) {
    __shared__ float As[2][TK + 2][LDA];  // rows TK, TK+1: landing area for the 32 threads without an A element
    __shared__ float Bs[2][TK][LDB];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int l16 = lane & 15, kq = lane >> 4;
    tile_id tile;
    int nk = (K + TK - 1) / TK;  // k tiles this block multiplies, starting at k tile kt0
    int kt0 = 0;
    float* piece_out = nullptr;
    if (FAST && split.pieces > 0) {
        const int xcd = blockIdx.x & 7, item = blockIdx.x >> 3;
        int v = xcd * split.per + item;
        if (item >= split.whole) {
            const int p = item - split.whole, cut = p / split.pieces, piece = p % split.pieces;
            v = xcd * split.per + split.whole + cut;
            kt0 = (int)((int64_t)nk * piece / split.pieces);
            nk = (int)((int64_t)nk * (piece + 1) / split.pieces) - kt0;
            piece_out = split.scratch +
                        ((int64_t)(xcd * (split.per - split.whole) + cut) * split.pieces + piece) * (TM * TN);
        }
        tile.x = v % split.gx;
        tile.y = (v / split.gx) % split.gy;
        tile.z = v / (split.gx * split.gy);
    } else {
        tile = xcd_tile();
    }
    const int m0 = tile.y * TM, n0 = tile.x * TN;
    A += (int64_t)(a_batch ? a_batch[tile.z] : tile.z) * strideA + (int64_t)kt0 * TK * lda;
    B += (int64_t)tile.z * strideB + (int64_t)kt0 * TK * ldb;
    C += (int64_t)(c_batch ? c_batch[tile.z] : tile.z) * strideC;

    v4acc acc[7][2];
#pragma unroll
    for (int i = 0; i < 7; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (v4acc)(0.0f);

    const bool a_inside = a_vec_ok && (m0 + TM <= M);
    const bool b_inside = b_vec_ok && (n0 + TN <= N);
    // A tile: 8 x 112 floats = 224 float4 (threads 0..223); B tile: 8 x 128 = 256 float4
    const bool a_thread = t < TK * (TM / 4);
    const int ak = a_thread ? t / (TM / 4) : 0, am4 = a_thread ? (t % (TM / 4)) * 4 : 0;
    const int bk = t >> 5, bn4 = (t & 31) * 4;
    // every thread loads and stores (threads 224..255 repeat element 0 of the A tile and park
    // it behind the tile), so neither the number of loads in flight nor the place of the
    // load in the instruction stream depends on the thread: a store under a per-thread
    // condition would pull its load in right before it
    float* a_dst = a_thread ? &As[0][ak][am4] : &As[0][TK][0] + (t - TK * (TM / 4)) * 4;
    // uniform base (row k0 of the operand) plus a 32-bit per-thread byte offset
    const uint32_t a_off = (uint32_t)(((int64_t)ak * lda + m0 + am4) * 4);
    const uint32_t b_off = (uint32_t)(((int64_t)bk * ldb + n0 + bn4) * 4);
    auto gload_fast = [&](int k0, v4f& ra, v4f& rb) {
        const char* abase = reinterpret_cast<const char*>(A + (int64_t)k0 * lda);
        const char* bbase = reinterpret_cast<const char*>(B + (int64_t)k0 * ldb);
        ra = *reinterpret_cast<const v4f*>(abase + a_off);
        rb = *reinterpret_cast<const v4f*>(bbase + b_off);
    };
    auto gload = [&](int k0, v4f& ra, v4f& rb) {
        const bool k_inside = k0 + TK <= K;
        ra = (v4f)(0.0f);
        if (a_thread) {
            const int gk = k0 + ak, gm = m0 + am4;
            const float* p = A + (int64_t)gk * lda + gm;
            if (a_inside && k_inside)
                ra = *reinterpret_cast<const v4f*>(p);
            else if (gk < K)
                ra = load4(p, (int64_t)M - gm, a_vec_ok);
        }
        const int gk = k0 + bk, gn = n0 + bn4;
        const float* q = B + (int64_t)gk * ldb + gn;
        if (b_inside && k_inside)
            rb = *reinterpret_cast<const v4f*>(q);
        else
            rb = (gk < K) ? load4(q, (int64_t)N - gn, b_vec_ok) : (v4f)(0.0f);
    };
    auto sstore = [&](int buf, const v4f& ra, const v4f& rb) {
        *reinterpret_cast<v4f*>(a_dst + buf * ((TK + 2) * LDA)) = ra;
        *reinterpret_cast<v4f*>(&Bs[buf][bk][bn4]) = rb;
    };
    auto compute = [&](int buf) {
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < TK / 4; ++ks) {
            const int k = 4 * ks + kq;
            const float b0 = Bs[buf][k][wave * 32 + l16];
            const float b1 = Bs[buf][k][wave * 32 + 16 + l16];
#pragma unroll
            for (int bm = 0; bm < 7; ++bm) {
                const float a = As[buf][k][bm * 16 + l16];
                acc[bm][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b0, acc[bm][0], 0, 0, 0);
                acc[bm][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b1, acc[bm][1], 0, 0, 0);
            }
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // two k tiles deep, as in mlp_gemm_kernel.  FAST (chosen by the host when every tile of
    // the launch is interior, 16-byte addressable and K a whole number of k tiles): loads
    // without guards and a steady-state loop without conditions, so that the wait before a
    // stage's LDS stores covers that stage's loads only.
    v4f pa, pb, qa, qb;
    int kt = 0;
    if (FAST) {
        // one register stage here: the accumulators leave room for no second one at five
        // blocks per CU, and a tile fetched at the start of a multiplication has all of it
        // (28 MFMAs per wave, five waves per SIMD) to arrive
        gload_fast(0, pa, pb);
        sstore(0, pa, pb);
        __syncthreads();
        // the scheduling barriers keep the loads where they are written, ahead of the
        // multiplication that hides them (left alone, the scheduler moves them down to
        // the wait in front of the LDS stores)
        for (; kt + 2 < nk; kt += 2) {
            gload_fast((kt + 1) * TK, pa, pb);
            __builtin_amdgcn_sched_barrier(0);
            compute(0);
            __builtin_amdgcn_sched_barrier(0);
            sstore(1, pa, pb);
            __syncthreads();
            gload_fast((kt + 2) * TK, pa, pb);
            __builtin_amdgcn_sched_barrier(0);
            compute(1);
            __builtin_amdgcn_sched_barrier(0);
            sstore(0, pa, pb);
            __syncthreads();
        }
        // one or two tiles left; buffer 0 holds tile kt
        if (kt + 1 < nk) gload_fast((kt + 1) * TK, pa, pb);
        compute(0);
        if (kt + 1 < nk) {
            sstore(1, pa, pb);
            __syncthreads();
            compute(1);
        }
    } else {
        gload(0, pa, pb);
        sstore(0, pa, pb);
        if (nk > 1) gload(TK, qa, qb);
        __syncthreads();
        for (; kt < nk; kt += 2) {
            if (kt + 2 < nk) gload((kt + 2) * TK, pa, pb);
            compute(0);
            if (kt + 1 < nk) sstore(1, qa, qb);
            __syncthreads();
            if (kt + 3 < nk) gload((kt + 3) * TK, qa, qb);
            if (kt + 1 < nk) compute(1);
            if (kt + 2 < nk) sstore(0, pa, pb);
            __syncthreads();
        }
    }

    // result block: register r of lane l is element (row 4*(l/16) + r, column l % 16)
    if (FAST) {   // every tile is interior; a piece of a tile goes to its scratch tile, rows of TN
        float* out = piece_out ? piece_out : C + (int64_t)m0 * ldc + n0;
        const int64_t ldo = piece_out ? TN : ldc;
        out += (int64_t)(4 * kq) * ldo + wave * 32 + l16;
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
            for (int bm = 0; bm < 7; ++bm)
#pragma unroll
                for (int r = 0; r < 4; ++r) out[(bm * 16 + r) * ldo + bn * 16] = acc[bm][bn][r];
        return;
    }
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
        const int gn = n0 + wave * 32 + bn * 16 + l16;
        if (gn >= N) continue;
#pragma unroll
        for (int bm = 0; bm < 7; ++bm) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int gm = m0 + bm * 16 + 4 * kq + r;
                if (gm < M) C[(int64_t)gm * ldc + gn] = acc[bm][bn][r];
            }
        }
    }
}

// The pieces of cut tile q of an evened-out launch, added in piece order and written to the
// tile's place in C; slab y (0..6) is rows 16y..16y+15, thread t takes four consecutive columns
// of rows 16y + t/32 and 16y + 8 + t/32.
__device__ __forceinline__ void join_tile(float* __restrict__ C, int64_t ldc, int64_t strideC,
                                          const int* __restrict__ c_batch, const k_split& split, int q,
                                          int y) {
    const int cuts = split.per - split.whole;
    const int xcd = q / cuts, cut = q % cuts;
    const int v = xcd * split.per + split.whole + cut;
    const int tx = v % split.gx, ty = (v / split.gx) % split.gy, tz = v / (split.gx * split.gy);
    const float* src = split.scratch + (int64_t)q * split.pieces * (TM * TN);
    float* dst = C + (int64_t)(c_batch ? c_batch[tz] : tz) * strideC + (int64_t)ty * TM * ldc + tx * TN;
    const int t = threadIdx.x;
    // both rows' pieces are asked for before any is added, eight pieces per row at a time: the
    // kernel is short and bound by how many loads it has in flight
    const int col = (t & 31) * 4;
    const int row[2] = {y * 16 + (t >> 5), y * 16 + 8 + (t >> 5)};
    v4f acc[2];
    for (int p0 = 0; p0 < split.pieces; p0 += 8) {  // block-uniform trip count
        v4f x[2][8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                if (p0 + u < split.pieces)
                    x[h][u] = *reinterpret_cast<const v4f*>(src + (int64_t)(p0 + u) * (TM * TN) + row[h] * TN + col);
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                if (p0 + u < split.pieces) acc[h] = (p0 + u == 0) ? x[h][u] : acc[h] + x[h][u];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float* o = dst + (int64_t)row[h] * ldc + col;
        o[0] = acc[h].x;
        o[1] = acc[h].y;
        o[2] = acc[h].z;
        o[3] = acc[h].w;
    }
}

template <int CTRL>
__device__ __forceinline__ float dpp_step(float v) {
    int iv = __builtin_bit_cast(int, v);
    int sh = __builtin_amdgcn_update_dpp(iv, iv, CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, sh);
}
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
    int iv = __builtin_bit_cast(int, v);
    int sh = __builtin_amdgcn_update_dpp(iv, iv, CTRL, 0xF, 0xF, false);
    return fmaxf(v, __builtin_bit_cast(float, sh));
}
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_step<0xB1>(v);
    v = dpp_step<0x4E>(v);
    v = dpp_step<0x141>(v);
    v = dpp_step<0x140>(v);
    int iv = __builtin_bit_cast(int, v);
    float s0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    float s1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    float s2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    float s3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return (s0 + s1) + (s2 + s3);
}

// Step 2a.  Logits, softmax and dZ2 = P - onehot(label), one lane per row so
// that no value crosses lanes inside a wave: a block takes 64 consecutive rows;
// their hidden activations pass through LDS in tiles of 64 rows x 32 units
// (coalesced 128-byte row segments in, one padded row per lane out), and each
// lane adds h * W2[unit][class] into its own NCP logits.  The 32 rows of W2
// that go with a tile sit in LDS as well and are read as broadcasts (every lane
// the same address).  The block's four waves share the hidden layer (wave w
// takes slices w, w+4, ... through a tile of its own; with one wave per block
// the launch had fewer waves than the chip has SIMDs) and their partial logits
// are added in wave order at the end.  The next tile is fetched into registers
// while the current one is consumed.  NCP is the class count rounded up;
// classes beyond `classes` get logit -inf.
// FAST: the class count is NCP itself, rows of H are 16-byte addressable and the hidden layer is
// a whole number of 128-unit rounds.  Then no load sits behind a condition (rows past the end
// are read from the last row and dropped), and the W2 rows, which are the same for every lane,
// come through wide scalar loads straight into the multiply-adds instead of being staged in
// LDS and read back as broadcasts (three quarters of the LDS reads of the other variant).
// Same order of additions either way.
template <int NCP, bool FAST>
__global__ __launch_bounds__(256) void mlp_logits_kernel(
    const float* __restrict__ H, const int* __restrict__ labels, const float* __restrict__ W2,
    const float* __restrict__ b2, float* __restrict__ dZ2, int hidden, int classes,
    int64_t total_rows, int h_vec_ok, int64_t rows, const int* __restrict__ unit_part) {
    constexpr int TR = 64, TH = 32, LD = TH + 4, NW = 4;
    constexpr int NCQ = (NCP + 3) / 4 * 4;  // W2 row padded to whole float4
    static_assert(NW * NCP * 64 <= NW * TR * LD, "the exchange of partial logits fits the tiles");
    __shared__ float tile_s[NW][TR * LD];
    // the fast variant keeps no W2 rows in LDS: 36 KiB per block, so that four blocks fit a CU and
    // the 64-row tiles of the usual batch sizes are all resident in one round
    __shared__ float w2s_s[FAST ? 1 : NW][FAST ? 4 : TH * NCQ];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* tile = tile_s[wave];
    float* w2s = w2s_s[FAST ? 0 : wave];
    const int64_t row0 = (int64_t)blockIdx.x * TR;
    const int64_t my_row = row0 + lane;
    float z[NCP];
#pragma unroll
    for (int q = 0; q < NCP; ++q) z[q] = 0.0f;

    // tile element idx = u*64 + lane: row idx/8, float4 idx%8
    v4f stage[8];
    float wstage[(TH * NCQ + 63) / 64];
    auto fetch = [&](int hc) {
        if (FAST) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = u * 64 + lane;
                int64_t r = row0 + (idx >> 3);
                r = r < total_rows ? r : total_rows - 1;
                stage[u] = *reinterpret_cast<const v4f*>(H + r * hidden + hc + (idx & 7) * 4);
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < (TH * NCQ + 63) / 64; ++u) {
            const int idx = u * 64 + lane;
            const int h = hc + idx / NCQ, q = idx % NCQ;
            wstage[u] = (idx < TH * NCQ && h < hidden && q < classes) ? W2[(int64_t)h * classes + q] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = u * 64 + lane;
            const int64_t r = row0 + (idx >> 3);
            const int h0 = hc + (idx & 7) * 4;
            stage[u] = r < total_rows ? load4(H + r * hidden + h0, (int64_t)hidden - h0, h_vec_ok)
                                      : (v4f)(0.0f);
        }
    };
    // the four waves take the 32-unit slices of the hidden layer in turn (wave w: slices w,
    // w+4, ...), each through its own tile; a slice past the end is skipped by its wave
    if (wave * TH < hidden) fetch(wave * TH);
    for (int hb = 0; hb < hidden; hb += NW * TH) {
        const int hc = hb + wave * TH;
        const bool live = hc < hidden;  // wave-uniform
        if (live) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = u * 64 + lane;
                *reinterpret_cast<v4f*>(&tile[(idx >> 3) * LD + (idx & 7) * 4]) = stage[u];
            }
            if (!FAST) {
#pragma unroll
                for (int u = 0; u < (TH * NCQ + 63) / 64; ++u) {
                    const int idx = u * 64 + lane;
                    if (idx < TH * NCQ) w2s[idx] = wstage[u];
                }
            }
        }
        // the tile and the W2 rows in LDS belong to this wave alone: its LDS writes and reads
        // execute in program order, no barrier is needed between them
        if (hc + NW * TH < hidden) fetch(hc + NW * TH);
        if (FAST) {
            const float* wslice = W2 + (int64_t)hc * NCP;  // wave-uniform: scalar loads
#pragma unroll
            for (int g = 0; g < TH / 4; ++g) {
                const v4f hv = *reinterpret_cast<const v4f*>(&tile[lane * LD + g * 4]);
                const float he[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int q = 0; q < NCP; ++q) z[q] += he[e] * wslice[(g * 4 + e) * NCP + q];
            }
        } else if (live) {
            // units past `hidden` carry zeros in both the tile and the W2 rows
#pragma unroll
            for (int g = 0; g < TH / 4; ++g) {
                const v4f hv = *reinterpret_cast<const v4f*>(&tile[lane * LD + g * 4]);
                const float he[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float* wrow = &w2s[(g * 4 + e) * NCQ];
#pragma unroll
                    for (int q4 = 0; q4 < NCQ / 4; ++q4) {
                        const v4f w = *reinterpret_cast<const v4f*>(wrow + q4 * 4);  // broadcast read
                        const float we[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (q4 * 4 + c < NCP) z[q4 * 4 + c] += he[e] * we[c];
                    }
                }
            }
        }
    }
    // the waves' partial logits meet in LDS, in the space of the tiles, once every wave is done
    // with its own, and wave 0 adds them in wave order: a fixed order, whatever the timing
    __syncthreads();
    float* zx = &tile_s[0][0];  // [NW][NCP][64]
#pragma unroll
    for (int q = 0; q < NCP; ++q) zx[(wave * NCP + q) * 64 + lane] = z[q];
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int q = 0; q < NCP; ++q) {
        float acc = zx[q * 64 + lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) acc += zx[(w * NCP + q) * 64 + lane];
        z[q] = acc;
    }
    if (my_row >= total_rows) return;
    // row r of H belongs to unit r / rows, which works on partition unit_part[unit]
    const int label = labels[unit_part ? (int64_t)unit_part[my_row / rows] * rows + my_row % rows : my_row];
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < NCP; ++q) {
        z[q] = q < classes ? z[q] + b2[q] : -INFINITY;
        mx = fmaxf(mx, z[q]);
    }
    float den = 0.0f;
#pragma unroll
    for (int q = 0; q < NCP; ++q) {
        z[q] = expf(z[q] - mx);
        den += z[q];
    }
    const float inv = 1.0f / den;
#pragma unroll
    for (int q = 0; q < NCP; ++q)
        if (q < classes) dZ2[my_row * classes + q] = z[q] * inv - (q == label ? 1.0f : 0.0f);
}

// Step 2b.  A block owns a run of rows of one partition and a slice of 1024 hidden
// units (blockIdx.y); thread t owns units 4t..4t+3 of the slice.  Per row it reads dZ2 (the same for the whole block), forms
// dH = dZ2 W2^T for its units, writes dZ1 = dH * [H > 0] over H and accumulates
// dW2 += h dZ2, db1 += dZ1, db2 += dZ2 in registers: no exchange between threads.
// Block partial layout = tail of theta: [db1 (hidden) | dW2 (hidden x classes) | db2 (classes)].
// FAST: the class count is NCP itself, rows of H are 16-byte addressable and every thread of
// the block owns four existing units (hidden a multiple of 1024).  Whole trips of RB rows then
// run without a condition around any load or store, so that each row's arithmetic waits for
// its own load only and the dZ2 values of a row arrive in wide scalar loads; what is left of
// the chunk, and every other shape, takes the guarded trip.  Same order of additions either way.
template <int NCP, bool FAST>
__global__ __launch_bounds__(256) void mlp_back_kernel(
    float* __restrict__ H, const float* __restrict__ dZ2, const float* __restrict__ W2,
    float* __restrict__ partial, int hidden, int classes, int64_t rows, int chunks,
    int64_t rows_per_chunk, int h_vec_ok) {
    const int t = threadIdx.x;
    const int j = blockIdx.x / chunks, c = blockIdx.x % chunks;
    const int64_t r0 = (int64_t)c * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const int h0 = 4 * t + 1024 * blockIdx.y;  // blockIdx.y: 1024-unit slice of the hidden layer
    const int hleft = hidden - h0;  // may be <= 0

    float w2[4][NCP], dw2[4][NCP], db1[4], db2[NCP];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        db1[e] = 0.0f;
#pragma unroll
        for (int q = 0; q < NCP; ++q) {
            w2[e][q] = (e < hleft && q < classes) ? W2[(int64_t)(h0 + e) * classes + q] : 0.0f;
            dw2[e][q] = 0.0f;
        }
    }
#pragma unroll
    for (int q = 0; q < NCP; ++q) db2[q] = 0.0f;

    float* Hp = H + ((int64_t)j * rows) * hidden + h0;
    const float* dzp = dZ2 + ((int64_t)j * rows) * classes;
    // one row: dz = its dZ2 values (block-uniform), hq = this thread's four activations
    auto one_row = [&](const float (&dz)[NCP], const v4f hq) -> v4f {
        const float hv[4] = {hq.x, hq.y, hq.z, hq.w};
        float dh[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int q = 0; q < NCP; ++q) {
            db2[q] += dz[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dw2[e][q] += hv[e] * dz[q];
                dh[e] += dz[q] * w2[e][q];
            }
        }
        v4f out;
        out.x = hv[0] > 0.0f ? dh[0] : 0.0f;  // ReLU'(0) = 0
        out.y = hv[1] > 0.0f ? dh[1] : 0.0f;
        out.z = hv[2] > 0.0f ? dh[2] : 0.0f;
        out.w = hv[3] > 0.0f ? dh[3] : 0.0f;
        db1[0] += out.x;
        db1[1] += out.y;
        db1[2] += out.z;
        db1[3] += out.w;
        return out;
    };
    // RB rows per trip: their loads are issued together before any is used
    constexpr int RB = 8;
    int64_t rb = r0;
    if (FAST) {
        for (; rb + RB <= r1; rb += RB) {
            v4f hq[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) hq[u] = *reinterpret_cast<const v4f*>(Hp + (rb + u) * hidden);
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                float dz[NCP];
#pragma unroll
                for (int q = 0; q < NCP; ++q) dz[q] = dzp[(rb + u) * NCP + q];  // block-uniform
                *reinterpret_cast<v4f*>(Hp + (rb + u) * hidden) = one_row(dz, hq[u]);
            }
        }
    }
    for (; rb < r1; rb += RB) {
        v4f hq[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int64_t r = rb + u < r1 ? rb + u : r1 - 1;
            hq[u] = load4(Hp + r * hidden, hleft, h_vec_ok);
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int64_t r = rb + u;
            if (r < r1) {  // block-uniform
                float* hrow = Hp + r * hidden;
                float dz[NCP];
#pragma unroll
                for (int q = 0; q < NCP; ++q) dz[q] = q < classes ? dzp[r * classes + q] : 0.0f;  // block-uniform
                const v4f out = one_row(dz, hq[u]);
                if (hleft >= 4 && h_vec_ok) {
                    *reinterpret_cast<v4f*>(hrow) = out;
                } else {
                    if (hleft > 0) hrow[0] = out.x;
                    if (hleft > 1) hrow[1] = out.y;
                    if (hleft > 2) hrow[2] = out.z;
                    if (hleft > 3) hrow[3] = out.w;
                }
            }
        }
    }
    const int64_t T = (int64_t)hidden + (int64_t)hidden * classes + classes;
    float* P = partial + (int64_t)blockIdx.x * T;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (e < hleft) {
            P[h0 + e] = db1[e];
#pragma unroll
            for (int q = 0; q < NCP; ++q)
                if (q < classes) P[hidden + (int64_t)(h0 + e) * classes + q] = dw2[e][q];
        }
    }
    if (t == 0 && blockIdx.y == 0) {
#pragma unroll
        for (int q = 0; q < NCP; ++q)
            if (q < classes) P[hidden + (int64_t)hidden * classes + q] = db2[q];
    }
}

// Steps 2a and 2b in one pass over H, for a hidden layer of exactly 1024 units and a class count
// equal to NCP: H is read once and dZ1 written once, no dZ2 array in between.  A block of 8
// waves owns a run of rows of one partition and takes them in trips of 8 rows; thread t owns
// units 2t, 2t+1, wave w units 128w..128w+127.  Per trip:
//   - the 8 rows go from registers into an LDS tile (row stride 1028 words: the eight rows a
//     16-byte LDS read touches lie in eight different bank groups);
//   - logits on the matrix cores (v_mfma_f32_16x16x4_f32, rows 8..15 of the 16-row block are
//     not used): wave w multiplies its 128 units of the tile by its 128 rows of W2, which it
//     holds in registers in operand layout for the whole kernel (lane l: class l % 16, unit
//     16 s + 4 (l / 16) + e of step s, component e); the eight partial logits per (row, class)
//     meet in LDS and are added in wave order;
//   - softmax and dZ2 = P - onehot(label) by 16 lanes per row (waves 0 and 1), into LDS;
//   - every thread reads the trip's dZ2 as LDS broadcasts and does what mlp_back_kernel does
//     for its two units: dH = dZ2 W2^T, dZ1 = dH * [H > 0] over H, dW2 += h dZ2, db1 += dZ1,
//     db2 += dZ2, in registers.
// The next trip's rows are fetched into a second register set before the arithmetic of this one.
// Block partial layout as in mlp_back_kernel.
template <int NCP>
__global__ __launch_bounds__(512, NCP <= 10 ? 4 : 2) void mlp_head1024_kernel(
    float* __restrict__ H, const int* __restrict__ labels, const float* __restrict__ W2,
    const float* __restrict__ b2, float* __restrict__ partial, int64_t rows, int chunks,
    int64_t rows_per_chunk, const int* __restrict__ unit_part) {
    constexpr int HID = 1024, TR = 8, LDH = HID + 4, NWV = 8;
    __shared__ __attribute__((aligned(16))) float hs[TR][LDH];
    __shared__ __attribute__((aligned(16))) float w2t[NCP][LDH];  // W2 transposed: [class][unit]
    __shared__ float zp[NWV][TR][16];
    __shared__ __attribute__((aligned(16))) float dzs[TR][16];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, kq = lane >> 4;
    const int j = blockIdx.x / chunks, c = blockIdx.x % chunks;
    const int64_t r0 = (int64_t)c * rows_per_chunk;
    const int64_t r1 = rows < r0 + rows_per_chunk ? rows : r0 + rows_per_chunk;
    const int h0 = 2 * t;

    float w2[2][NCP], dw2[2][NCP], db1[2] = {0.0f, 0.0f};
    float db2 = 0.0f;  // threads 0..127: the sum of dZ2 over the rows (trip row t / 16, class t % 16) they handle
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int q = 0; q < NCP; ++q) {
            w2[e][q] = W2[(int64_t)(h0 + e) * NCP + q];
            dw2[e][q] = 0.0f;
        }
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int q = 0; q < NCP; ++q) w2t[q][h0 + e] = w2[e][q];

    float* Hp = H + ((int64_t)j * rows) * HID + h0;
    const int* lab = labels + (int64_t)(unit_part ? unit_part[j] : j) * rows;
    // rows past the end of the chunk are read from its last row and dropped
    auto fetch = [&](int64_t rb, v2f (&hq)[TR]) {
#pragma unroll
        for (int u = 0; u < TR; ++u) {
            const int64_t r = rb + u < r1 ? rb + u : r1 - 1;
            hq[u] = *reinterpret_cast<const v2f*>(Hp + r * HID);
        }
    };
    // the softmax lanes (threads 0..127: trip row t / 16, class t % 16) hold their class's bias for the
    // whole kernel and ask for a trip's label together with its rows, a trip ahead: the softmax step
    // keeps all eight waves waiting and must not begin with a trip to memory
    const int srow = t >> 4, sq = t & 15;
    const float b2q = (t < TR * 16 && sq < NCP) ? b2[sq] : 0.0f;
    auto fetch_label = [&](int64_t rb) {
        const int64_t r = rb + srow < r1 ? rb + srow : r1 - 1;
        return t < TR * 16 ? lab[r] : 0;
    };
    v2f hq[TR], nq[TR];
    int label = 0, label_n = 0;
    if (r0 < r1) {
        fetch(r0, hq);
        label = fetch_label(r0);
    }
    for (int64_t rb = r0; rb < r1; rb += TR) {
#pragma unroll
        for (int u = 0; u < TR; ++u) *reinterpret_cast<v2f*>(&hs[u][h0]) = hq[u];
        __syncthreads();
        if (rb + TR < r1) {
            fetch(rb + TR, nq);
            label_n = fetch_label(rb + TR);
        }
        {   // partial logits of the wave's 128 units
            // four accumulators, one per component, so that no product waits for the one before
            // it; added in component order at the end
            v4acc acc0 = (v4acc)(0.0f), acc1 = (v4acc)(0.0f), acc2 = (v4acc)(0.0f), acc3 = (v4acc)(0.0f);
            // first operand: lane l feeds (row l % 16, unit 16 s + 4 (l / 16) + e), second operand
            // (unit the same, class l % 16).  Rows 8..15 repeat rows 0..7 and classes >= NCP repeat
            // lower ones: their results land in rows and columns of the block that nobody reads
            const float* arow = &hs[l16 & (TR - 1)][wave * 128 + 4 * kq];
            const float* brow = &w2t[l16 % NCP][wave * 128 + 4 * kq];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const v4f a4 = *reinterpret_cast<const v4f*>(arow + 16 * s);
                const v4f b4 = *reinterpret_cast<const v4f*>(brow + 16 * s);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, b4.x, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, b4.y, acc1, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, b4.z, acc2, 0, 0, 0);
                acc3 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, b4.w, acc3, 0, 0, 0);
            }
            const v4acc acc = (acc0 + acc1) + (acc2 + acc3);
            // result block: register r of lane l is (row 4 (l / 16) + r, class l % 16); rows 0..7 exist
            if (kq < 2) {
#pragma unroll
                for (int r = 0; r < 4; ++r) zp[wave][4 * kq + r][l16] = acc[r];
            }
        }
        __syncthreads();
        if (t < TR * 16) {   // waves 0 and 1: 16 lanes per row
            const int row = srow, q = sq;
            float z = -INFINITY;
            if (q < NCP) {
                z = zp[0][row][q];
#pragma unroll
                for (int w = 1; w < NWV; ++w) z += zp[w][row][q];
                z += b2q;
            }
            // maximum and sum over the 16 lanes of the row, every lane gets both (data-parallel
            // moves within quads, half rows and rows; fixed order)
            float mx = z;
            mx = dpp_max<0xB1>(mx);
            mx = dpp_max<0x4E>(mx);
            mx = dpp_max<0x141>(mx);
            mx = dpp_max<0x140>(mx);
            const float ez = q < NCP ? expf(z - mx) : 0.0f;
            float den = ez;
            den = dpp_step<0xB1>(den);
            den = dpp_step<0x4E>(den);
            den = dpp_step<0x141>(den);
            den = dpp_step<0x140>(den);
            const float dz = q < NCP ? ez * (1.0f / den) - (q == label ? 1.0f : 0.0f) : 0.0f;
            dzs[row][q] = dz;
            if (rb + row < r1) db2 += dz;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < TR; ++u) {
            if (rb + u < r1) {   // block-uniform
                float dz[NCP];
#pragma unroll
                for (int q = 0; q < NCP; ++q) dz[q] = dzs[u][q];  // the same address in every lane
                const float hv[2] = {hq[u].x, hq[u].y};
                float dh[2] = {0.0f, 0.0f};
#pragma unroll
                for (int q = 0; q < NCP; ++q) {
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        dw2[e][q] += hv[e] * dz[q];
                        dh[e] += dz[q] * w2[e][q];
                    }
                }
                v2f out;
                out.x = hv[0] > 0.0f ? dh[0] : 0.0f;  // ReLU'(0) = 0
                out.y = hv[1] > 0.0f ? dh[1] : 0.0f;
                db1[0] += out.x;
                db1[1] += out.y;
                *reinterpret_cast<v2f*>(Hp + (rb + u) * HID) = out;
            }
        }
#pragma unroll
        for (int u = 0; u < TR; ++u) hq[u] = nq[u];
        label = label_n;
    }
    const int64_t T = (int64_t)HID + (int64_t)HID * NCP + NCP;
    float* P = partial + (int64_t)blockIdx.x * T;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        P[h0 + e] = db1[e];
#pragma unroll
        for (int q = 0; q < NCP; ++q) P[HID + (int64_t)(h0 + e) * NCP + q] = dw2[e][q];
    }
    // db2: the eight row slots of a class are added in slot order
    __syncthreads();
    if (t < TR * 16) dzs[t >> 4][t & 15] = db2;
    __syncthreads();
    if (t < NCP) {
        float acc = dzs[0][t];
#pragma unroll
        for (int u = 1; u < TR; ++u) acc += dzs[u][t];
        P[HID + (int64_t)HID * NCP + t] = acc;
    }
}

// The fixed-order sums that close a gradient call, one launch.  Blocks below join_blocks add
// the pieces of the backward product's cut tiles (block b: tile b / 7, slab b % 7; none unless
// the product was evened out).  The others sum the head's block partials: block b' = b -
// join_blocks takes unit j = b' / tail_blocks and elements 256 (b' % tail_blocks)..+255:
// out[row(j)*out_stride + t] = sum over chunks (in index order) of partial[(j*chunks + c)*T + t],
// row(j) = unit_row[j], or j without a map.
__global__ __launch_bounds__(256) void mlp_sums_kernel(int join_blocks, float* __restrict__ C, int64_t ldc,
                                                       int64_t strideC, const k_split split,
                                                       const float* __restrict__ partial,
                                                       float* __restrict__ out, int64_t T, int chunks,
                                                       int tail_blocks, int64_t out_stride,
                                                       const int* __restrict__ unit_row) {
    if ((int)blockIdx.x < join_blocks) {
        join_tile(C, ldc, strideC, unit_row, split, blockIdx.x / (TM / 16), blockIdx.x % (TM / 16));
        return;
    }
    const int b = blockIdx.x - join_blocks;
    const int j = b / tail_blocks;
    const int64_t t = (int64_t)(b % tail_blocks) * 256 + threadIdx.x;
    if (t >= T) return;
    const float* p = partial + (int64_t)j * chunks * T + t;
    float acc = 0.0f;
    for (int c0 = 0; c0 < chunks; c0 += 32) {  // up to thirty-two loads in flight, added in index order
        float a[32];
#pragma unroll
        for (int u = 0; u < 32; ++u)
            if (c0 + u < chunks) a[u] = p[(int64_t)(c0 + u) * T];  // block-uniform condition
#pragma unroll
        for (int u = 0; u < 32; ++u)
            if (c0 + u < chunks) acc = (c0 + u == 0) ? a[u] : acc + a[u];
    }
    out[(int64_t)(unit_row ? unit_row[j] : j) * out_stride + t] = acc;
}

struct mlp_prof {
    ngc_ctx* ctx;
    hipEvent_t stop = nullptr;
    bool on = false;
    explicit mlp_prof(ngc_ctx* c) : ctx(c) {
        if (!((c->profile_mask >> NGC_KERNEL_MLP) & 1u) || c->prof.size() >= (size_t)NGC_MAX_PROFILE) return;
        ngc_profile_rec r;
        r.kernel = NGC_KERNEL_MLP;
        if (hipEventCreate(&r.start) != hipSuccess) return;
        if (hipEventCreate(&r.stop) != hipSuccess) {
            (void)hipEventDestroy(r.start);
            return;
        }
        (void)hipEventRecord(r.start, c->stream);
        stop = r.stop;
        c->prof.push_back(r);
        on = true;
    }
    ~mlp_prof() {
        if (on) (void)hipEventRecord(stop, ctx->stream);
    }
};

bool al(const void* p, uintptr_t m) { return (reinterpret_cast<uintptr_t>(p) & (m - 1)) == 0; }

}  // namespace

// Perceptron gradients of `units` partial-gradient computations.  Unit q works on partition
// unit_part[q] (q itself if the map is null) and its gradient goes to row unit_row[q] of G
// (row q if null); both maps are device arrays.  Without maps the units are the k partitions.
int ngc_mlp2_grads(ngc_ctx* ctx, const float* X, const int* labels, const float* theta,
                   int64_t rows, float* G, int units, const int* unit_part, const int* unit_row) {
    const int k = units;
    const int din = ctx->mlp_din, hid = ctx->mlp_hidden, cls = ctx->mlp_classes;
    const int64_t d = ctx->d;
    if (hid > 65535 * 1024) return ngc_fail(ctx, NGC_ERR_INVALID, "MLP hidden width too large");
    if (cls > 16) return ngc_fail(ctx, NGC_ERR_INVALID, "MLP with more than 16 classes is not supported");
    const int64_t total = (int64_t)k * rows;
    if (total > 0x7fffffffLL) return ngc_fail(ctx, NGC_ERR_INVALID, "too many rows");
    const float* W1 = theta;
    const float* b1 = theta + (int64_t)din * hid;
    const float* W2 = b1 + hid;
    const float* b2 = W2 + (int64_t)hid * cls;
    const int64_t T = (int64_t)hid + (int64_t)hid * cls + cls;

    // workspace: H [total][hid] | dZ2 [total][cls] | block partials [k*chunks][T]
    // blocks of the backward head kernel: as many as are resident at once (its register count
    // allows 5, 3 or 2 blocks per CU for up to 4, 10 or 16 classes), so there is no second round
    // (the one-pass head for 1024 hidden units: two blocks of 512 threads per CU, one at 16 classes)
    const bool head_fused = hid == 1024 && (cls == 4 || cls == 10 || cls == 16);
    const int back_per_cu = head_fused ? (cls == 16 ? 1 : 2) : (cls <= 4 ? 5 : (cls <= 10 ? 3 : 2));
    const int64_t slices = (hid + 1023) / 1024;  // the backward head kernel covers 1024 hidden units per block
    int64_t chunks = std::max<int64_t>(1, (int64_t)ctx->cu_count * back_per_cu / (k * slices));
    int64_t rpc = (rows + chunks - 1) / chunks;
    chunks = (rows + rpc - 1) / rpc;
    const size_t h_floats = (((size_t)total * hid) + 63) / 64 * 64;
    const size_t z_floats = (((size_t)total * cls) + 63) / 64 * 64;
    // backward product in tiles of 112 rows: if its tile count leaves some CUs one tile short of
    // the others, the last tiles of each XCD's run are cut along K (see k_split)
    const int64_t gemm_tiles = (int64_t)((hid + TN - 1) / TN) * ((din + TM - 1) / TM) * k;
    const int cus_per_xcd = ctx->cu_count / 8;
    int64_t gemm_cuts = 0;  // cut tiles per XCD
    int gemm_pieces = 8;    // pieces per cut tile: the fewest (4..16) that share out evenly over the XCD's CUs
    if (cus_per_xcd > 0 && gemm_tiles % 8 == 0 && gemm_tiles / 8 < 16 * (int64_t)cus_per_xcd) {
        gemm_cuts = (gemm_tiles / 8) % cus_per_xcd;
        for (int p = 4; p <= 16; ++p)
            if ((gemm_cuts * p) % cus_per_xcd == 0) {
                gemm_pieces = p;
                break;
            }
        if (rows / TK < 16 * gemm_pieces) gemm_cuts = 0;  // pieces of fewer than 16 k tiles are not worth their prologue
    }
    const size_t need = sizeof(float) * (h_floats + z_floats + (size_t)k * chunks * T +
                                         (size_t)(8 * gemm_cuts * gemm_pieces) * TM * TN);
    if (need > ctx->d_ws_bytes) {
        if (ctx->d_ws) {
            NGC_HIP(ctx, hipStreamSynchronize(ctx->stream));
            NGC_HIP(ctx, hipFree(ctx->d_ws));
            ctx->d_ws = nullptr;
            ctx->d_ws_bytes = 0;
        }
        void* p = nullptr;
        if (hipMalloc(&p, need) != hipSuccess) {
            (void)hipGetLastError();
            return ngc_fail(ctx, NGC_ERR_NOMEM, "workspace allocation failed");
        }
        ctx->d_ws = (float*)p;
        ctx->d_ws_bytes = need;
    }
    float* H = ctx->d_ws;
    float* dZ2 = ctx->d_ws + h_floats;
    float* partial = dZ2 + z_floats;

    mlp_prof ps(ctx);
    if (!unit_part) {   // 1. H = relu(X W1 + b1), all partitions as one matrix
        dim3 grid((unsigned)((hid + BN - 1) / BN), (unsigned)((total + BM - 1) / BM), 1);
        if (grid.y > 65535) return ngc_fail(ctx, NGC_ERR_INVALID, "too many rows for one launch");
        hipLaunchKernelGGL((mlp_gemm_kernel<false, EPI_BIAS_RELU>), grid, dim3(256), 0, ctx->stream, X, W1, H, b1,
                           (int)total, hid, din, (int64_t)din, (int64_t)hid, (int64_t)hid, (int64_t)0,
                           (int64_t)0, (int64_t)0, (int)(din % 4 == 0 && al(X, 16)),
                           (int)(hid % 4 == 0 && al(W1, 16)), (int)(hid % 2 == 0), (const int*)nullptr,
                           (const int*)nullptr);
        NGC_HIP(ctx, hipGetLastError());
    } else {   // the same, one batch entry per unit: entry q reads partition unit_part[q], writes H block q
        dim3 grid((unsigned)((hid + BN - 1) / BN), (unsigned)((rows + BM - 1) / BM), (unsigned)k);
        if (grid.y > 65535 || k > 65535) return ngc_fail(ctx, NGC_ERR_INVALID, "too many rows or units for one launch");
        hipLaunchKernelGGL((mlp_gemm_kernel<false, EPI_BIAS_RELU>), grid, dim3(256), 0, ctx->stream, X, W1, H, b1,
                           (int)rows, hid, din, (int64_t)din, (int64_t)hid, (int64_t)hid, rows * (int64_t)din,
                           (int64_t)0, rows * (int64_t)hid,
                           (int)(din % 4 == 0 && al(X, 16) && (rows * (int64_t)din) % 4 == 0),
                           (int)(hid % 4 == 0 && al(W1, 16)), (int)(hid % 2 == 0), unit_part,
                           (const int*)nullptr);
        NGC_HIP(ctx, hipGetLastError());
    }
    {   // 2. logits, softmax, dZ2; then dW2/db2/db1 partials and dZ1 over H
        const int hv = hid % 4 == 0;
        dim3 lgrid((unsigned)((total + 63) / 64));
        dim3 grid((unsigned)(k * chunks), (unsigned)((hid + 1023) / 1024));  // y: 1024-unit hidden slices
#define NGC_MLP_HEAD(NCP)                                                                              \
    if (hv && hid % 128 == 0 && cls == NCP)                                                            \
        hipLaunchKernelGGL((mlp_logits_kernel<NCP, true>), lgrid, dim3(256), 0, ctx->stream, (const float*)H, \
                           labels, W2, b2, dZ2, hid, cls, total, hv, rows, unit_part);                 \
    else                                                                                               \
        hipLaunchKernelGGL((mlp_logits_kernel<NCP, false>), lgrid, dim3(256), 0, ctx->stream, (const float*)H, \
                           labels, W2, b2, dZ2, hid, cls, total, hv, rows, unit_part);                 \
    if (hv && hid % 1024 == 0 && cls == NCP)                                                           \
        hipLaunchKernelGGL((mlp_back_kernel<NCP, true>), grid, dim3(256), 0, ctx->stream, H, (const float*)dZ2, \
                           W2, partial, hid, cls, rows, (int)chunks, rpc, hv);                         \
    else                                                                                               \
        hipLaunchKernelGGL((mlp_back_kernel<NCP, false>), grid, dim3(256), 0, ctx->stream, H, (const float*)dZ2, \
                           W2, partial, hid, cls, rows, (int)chunks, rpc, hv);
        if (head_fused) {
            dim3 fgrid((unsigned)(k * chunks));
            if (cls == 4)
                hipLaunchKernelGGL(mlp_head1024_kernel<4>, fgrid, dim3(512), 0, ctx->stream, H, labels, W2, b2, partial,
                                   rows, (int)chunks, rpc, unit_part);
            else if (cls == 10)
                hipLaunchKernelGGL(mlp_head1024_kernel<10>, fgrid, dim3(512), 0, ctx->stream, H, labels, W2, b2, partial,
                                   rows, (int)chunks, rpc, unit_part);
            else
                hipLaunchKernelGGL(mlp_head1024_kernel<16>, fgrid, dim3(512), 0, ctx->stream, H, labels, W2, b2, partial,
                                   rows, (int)chunks, rpc, unit_part);
        } else if (cls <= 4) {
            NGC_MLP_HEAD(4)
        } else if (cls <= 10) {
            NGC_MLP_HEAD(10)
        } else {
            NGC_MLP_HEAD(16)
        }
#undef NGC_MLP_HEAD
        NGC_HIP(ctx, hipGetLastError());
    }
    int join_blocks = 0;
    k_split split = {0, 0, 0, 0, 0, nullptr};
    {   // 3. dW1_j = X_j^T dZ1_j, one batch entry per partition, straight into G[j]
        const int a_ok = (int)(din % 4 == 0 && al(X, 16)), b_ok = (int)(hid % 4 == 0);
        // tiles of 112 rows when they pad the d_in rows less than tiles of 128 (784 = 7 * 112)
        const int64_t pad128 = (int64_t)((din + BM - 1) / BM) * BM, pad112 = (int64_t)((din + TM - 1) / TM) * TM;
        if (pad112 < pad128) {
            dim3 grid((unsigned)((hid + TN - 1) / TN), (unsigned)((din + TM - 1) / TM), (unsigned)k);
            const bool all_fast = a_ok && b_ok && din % TM == 0 && hid % TN == 0 && rows % TK == 0;
            split.gx = (int)grid.x;
            split.gy = (int)grid.y;
            if (all_fast && gemm_cuts > 0) {
                split.pieces = gemm_pieces;
                split.per = (int)(gemm_tiles / 8);
                split.whole = split.per - (int)gemm_cuts;
                split.scratch = partial + (size_t)k * chunks * T;
                hipLaunchKernelGGL(mlp_gemm112_kernel<true>, dim3((unsigned)(8 * (split.whole + gemm_cuts * gemm_pieces))),
                                   dim3(256), 0, ctx->stream, X, (const float*)H, G, din, hid, (int)rows,
                                   (int64_t)din, (int64_t)hid, (int64_t)hid, rows * (int64_t)din,
                                   rows * (int64_t)hid, d, a_ok, b_ok, unit_part, unit_row, split);
                join_blocks = (int)(8 * gemm_cuts) * (TM / 16);
            } else if (all_fast)
                hipLaunchKernelGGL(mlp_gemm112_kernel<true>, grid, dim3(256), 0, ctx->stream, X, (const float*)H, G,
                                   din, hid, (int)rows, (int64_t)din, (int64_t)hid, (int64_t)hid,
                                   rows * (int64_t)din, rows * (int64_t)hid, d, a_ok, b_ok, unit_part, unit_row, split);
            else
                hipLaunchKernelGGL(mlp_gemm112_kernel<false>, grid, dim3(256), 0, ctx->stream, X, (const float*)H, G,
                                   din, hid, (int)rows, (int64_t)din, (int64_t)hid, (int64_t)hid,
                                   rows * (int64_t)din, rows * (int64_t)hid, d, a_ok, b_ok, unit_part, unit_row, split);
        } else {
            dim3 grid((unsigned)((hid + BN - 1) / BN), (unsigned)((din + BM - 1) / BM), (unsigned)k);
            hipLaunchKernelGGL((mlp_gemm_kernel<true, EPI_STORE>), grid, dim3(256), 0, ctx->stream, X, (const float*)H, G,
                               (const float*)nullptr, din, hid, (int)rows, (int64_t)din, (int64_t)hid, (int64_t)hid,
                               rows * (int64_t)din, rows * (int64_t)hid, d, a_ok, b_ok,
                               (int)(hid % 2 == 0 && d % 2 == 0 && al(G, 8)), unit_part, unit_row);
        }
        NGC_HIP(ctx, hipGetLastError());
    }
    {   // 4. the sums that are left: pieces of cut tiles into G, the head's block partials into the tail of G
        const int tail_blocks = (int)((T + 255) / 256);
        hipLaunchKernelGGL(mlp_sums_kernel, dim3((unsigned)(join_blocks + tail_blocks * k)), dim3(256), 0, ctx->stream,
                           join_blocks, G, (int64_t)hid, d, split, (const float*)partial, G + (int64_t)din * hid, T,
                           (int)chunks, tail_blocks, d, unit_row);
        NGC_HIP(ctx, hipGetLastError());
    }
    return NGC_OK;
}
