// Backward pass of a GNN layer (the paper's training runs reuse the aggregation kernel on
// gradients, Sec. 7.2 "Training Support"): activation mask, bias gradient, weight gradient
// (a transposed tall-skinny GEMM reduced over the nodes), input gradient, and the aggregation of
// gradients over the transposed graph.
#include <hip/hip_runtime.h>

#include "gnn_launch.h"

namespace gnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTnBlocks = 256;  // row chunks of the transposed GEMM (one per CU)
constexpr int kTnWaves = 4;
constexpr int kTnPartials = kTnBlocks * kTnWaves;
constexpr int kBfBlocks = 512;  // row chunks of the one-pass kernel (two blocks per CU)
constexpr int kBfWaves = 4;
constexpr int kBfPartials = kBfBlocks * kBfWaves;
constexpr int kBfLd = 68;       // floats per LDS row of 64 (16-byte reads of a column block stay conflict-poor)
constexpr int kRedGroups = 32;  // first level of the sum over partial arrays
constexpr int kColsumBlocks = 1024;  // row chunks of the bias gradient

// dZ = dY where the forward output was positive, else 0 (derivative of ReLU through its output).
__global__ __launch_bounds__(256) void k_relu_mask(int64_t total, const float *__restrict__ dY,
                                                   const float *__restrict__ Y, float *__restrict__ dZ)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        dZ[i] = Y[i] > 0.0f ? dY[i] : 0.0f;
}

// Column sums of G[n,M], stage 1: block b sums its row chunk into part[b][M].  The 256 threads share the
// columns (up to 256 at a time) and, where there are fewer columns than threads, the rows: thread t takes column
// t % width and the rows r0 + t / width, + 256 / width, ...; the row lanes' sums meet in LDS in a fixed order.
__global__ __launch_bounds__(256) void k_colsum_partial(int n, int M, const float *__restrict__ G, float *__restrict__ part)
{
    __shared__ float red[256];
    const int64_t rows = ((int64_t)n + gridDim.x - 1) / gridDim.x;
    const int64_t r0 = (int64_t)blockIdx.x * rows;
    const int64_t r1 = r0 + rows < n ? r0 + rows : n;
    for (int c0 = 0; c0 < M; c0 += 256) {
        const int width = M - c0 < 256 ? M - c0 : 256;
        const int lanes = 256 / width;
        const int c = threadIdx.x % width, rs = threadIdx.x / width;
        float s = 0.0f;
        if (rs < lanes) {
#pragma unroll 4
            for (int64_t r = r0 + rs; r < r1; r += lanes) s += G[(size_t)r * M + c0 + c];
        }
        red[threadIdx.x] = s;
        __syncthreads();
        if ((int)threadIdx.x < width) {
            float t = 0.0f;
            for (int j = 0; j < lanes; ++j) t += red[j * width + threadIdx.x];
            part[(size_t)blockIdx.x * M + c0 + threadIdx.x] = t;
        }
        __syncthreads();
    }
}

// Sums groups of `count` consecutive partial arrays of `len` floats:
// out[g][i] = sum_{p < count} part[g*count + p][i], g = blockIdx.y.
__global__ __launch_bounds__(256) void k_reduce_partials(int count, int64_t len, const float *__restrict__ part,
                                                         float *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= len) return;
    const float *src = part + (size_t)blockIdx.y * count * len;
    float s = 0.0f;
#pragma unroll 8
    for (int p = 0; p < count; ++p) s += src[(size_t)p * len + i];
    out[(size_t)blockIdx.y * len + i] = s;
}

// Wt[M,K] = W[K,M]^T (small)
__global__ __launch_bounds__(256) void k_transpose(int K, int M, const float *__restrict__ W, float *__restrict__ Wt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K * M) {
        const int k = i / M, m = i % M;
        Wt[(size_t)m * K + k] = W[i];
    }
}

// C[K,M] = P[n,K]^T Q[n,M], stage 1.  A wave owns KT x MT tiles of 16x16 of the result (offset by
// blockIdx.y) and walks over its share of the rows four at a time: with v_mfma_f32_16x16x4_f32 the
// reduction index is the row, so both operands are read straight from global memory, 16 consecutive
// floats of 4 consecutive rows per instruction.  Every wave writes its partial result; stage 2 sums.
template <int KT, int MT>
__global__ __launch_bounds__(256) void k_gemm_tn_partial(int n, int K, int M, const float *__restrict__ P,
                                                         const float *__restrict__ Q, float *__restrict__ part,
                                                         int mgroups)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 15, lk = lane >> 4;
    const int kg = blockIdx.y / mgroups, mg = blockIdx.y % mgroups;
    const int k0 = kg * 16 * KT, m0 = mg * 16 * MT;
    constexpr int kSteps = 4;  // 4-row MFMA steps whose loads are issued together
    const int64_t rows = (((int64_t)n + gridDim.x - 1) / gridDim.x + 4 * kSteps - 1) / (4 * kSteps) * (4 * kSteps);
    const int64_t r0 = (int64_t)blockIdx.x * rows;
    const int64_t r1 = r0 + rows < n ? r0 + rows : n;

    f32x4 acc[KT][MT];
#pragma unroll
    for (int a = 0; a < KT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

    for (int64_t r = r0 + 4 * kSteps * wave; r < r1; r += 4 * kSteps * kTnWaves) {
        float av[kSteps][KT], bv[kSteps][MT];
#pragma unroll
        for (int u = 0; u < kSteps; ++u) {
            const int64_t row = r + 4 * u + lk;
            const bool rv = row < r1;
#pragma unroll
            for (int a = 0; a < KT; ++a) {
                const int k = k0 + a * 16 + lrow;
                av[u][a] = (rv && k < K) ? P[(size_t)row * K + k] : 0.0f;
            }
#pragma unroll
            for (int b = 0; b < MT; ++b) {
                const int m = m0 + b * 16 + lrow;
                bv[u][b] = (rv && m < M) ? Q[(size_t)row * M + m] : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < kSteps; ++u)
#pragma unroll
            for (int a = 0; a < KT; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][a], bv[u][b], acc[a][b], 0, 0, 0);
    }

    // lane holds result rows 4*(lane/16)+i, column lane%16 of each tile
    float *mine = part + ((size_t)blockIdx.x * kTnWaves + wave) * (size_t)K * M;
#pragma unroll
    for (int a = 0; a < KT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + a * 16 + 4 * lk + i, m = m0 + b * 16 + lrow;
                if (k < K && m < M) mine[(size_t)k * M + m] = acc[a][b][i];
            }
}

// Same product with 16-byte loads, for K and M multiples of 4: a lane reads P[row][k0 + 4*lrow .. +3]
// once and feeds its four values to four different result tiles, so tile a holds the result rows
// k0 + 4*i + a (i = 0..15) instead of 16 consecutive ones; likewise tile b holds the columns
// m0 + 4*j + b.  One pair of loads per 16 MFMAs, whole 256-byte row segments per instruction.
__global__ __launch_bounds__(256) void k_gemm_tn_partial_v4(int n, int K, int M, const float *__restrict__ P,
                                                            const float *__restrict__ Q, float *__restrict__ part,
                                                            int mgroups)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 15, lk = lane >> 4;
    const int kg = blockIdx.y / mgroups, mg = blockIdx.y % mgroups;
    const int k0 = kg * 64, m0 = mg * 64;
    constexpr int kSteps = 4;  // 4-row MFMA steps whose loads are issued together
    const int64_t rows = (((int64_t)n + gridDim.x - 1) / gridDim.x + 4 * kSteps - 1) / (4 * kSteps) * (4 * kSteps);
    const int64_t r0 = (int64_t)blockIdx.x * rows;
    const int64_t r1 = r0 + rows < n ? r0 + rows : n;
    const bool kin = k0 + 4 * lrow < K, min_ = m0 + 4 * lrow < M;

    f32x4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

    for (int64_t r = r0 + 4 * kSteps * wave; r < r1; r += 4 * kSteps * kTnWaves) {
        float4 pa[kSteps], qb[kSteps];
#pragma unroll
        for (int u = 0; u < kSteps; ++u) {
            const int64_t row = r + 4 * u + lk;
            const bool rv = row < r1;
            pa[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            qb[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rv && kin) pa[u] = *reinterpret_cast<const float4 *>(P + (size_t)row * K + k0 + 4 * lrow);
            if (rv && min_) qb[u] = *reinterpret_cast<const float4 *>(Q + (size_t)row * M + m0 + 4 * lrow);
        }
#pragma unroll
        for (int u = 0; u < kSteps; ++u) {
            const float av[4] = {pa[u].x, pa[u].y, pa[u].z, pa[u].w}, bv[4] = {qb[u].x, qb[u].y, qb[u].z, qb[u].w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
    }

    float *mine = part + ((size_t)blockIdx.x * kTnWaves + wave) * (size_t)K * M;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // MFMA result row 4*lk + i of tile a is k-index k0 + 4*(4*lk + i) + a; column lrow of tile b is m0 + 4*lrow + b
                const int k = k0 + 4 * (4 * lk + i) + a, m = m0 + 4 * lrow + b;
                if (k < K && m < M) mine[(size_t)k * M + m] = acc[a][b][i];
            }
}

// The whole backward of an Update in one pass over the rows, for widths of at most 64 that are multiples of 4:
//   G = dY where Y > 0 (MASK) or dY;   dW = P^T G;   db = column sums of G;   R = G W^T.
// A wave takes 16 rows at a time.  It loads P, dY (and Y) as the transposed product wants them (a lane: four
// consecutive columns of the rows 4u + lane/16), runs that product's 64 MFMAs, hands G through a private LDS tile
// to the layout of the second product (a lane: row lane%16, columns 16*(lane/16) .. +15) and computes R^T = W G^T
// with W (zero-padded to 64 x 64) read from LDS, so that a lane ends up with four consecutive columns of one
// row of R.  G is never written to memory: 3 reads and 1 write of n x 64 floats instead of 7 and 3.
// Every wave writes its partial dW (and db); the sums over waves are taken afterwards, in a fixed order.
template <bool MASK, bool WANT_R>
__global__ __launch_bounds__(256) void k_bwd_update_fused(int n, int K, int M, const float *__restrict__ P,
                                                          const float *__restrict__ dY, const float *__restrict__ Y,
                                                          const float *__restrict__ W, float *__restrict__ R,
                                                          float *__restrict__ part_w, float *__restrict__ part_b)
{
    __shared__ __attribute__((aligned(16))) float sW[WANT_R ? 64 * kBfLd : 4];
    __shared__ __attribute__((aligned(16))) float sG[kBfWaves][WANT_R ? 16 * kBfLd : 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 15, lk = lane >> 4;
    if (WANT_R) {
        for (int i = threadIdx.x; i < 64 * 64; i += 256) {
            const int k = i >> 6, m = i & 63;
            sW[k * kBfLd + m] = (k < K && m < M) ? W[(size_t)k * M + m] : 0.0f;
        }
        __syncthreads();
    }

    const int64_t rows = (((int64_t)n + gridDim.x - 1) / gridDim.x + 16 * kBfWaves - 1) / (16 * kBfWaves) * (16 * kBfWaves);
    const int64_t r0 = (int64_t)blockIdx.x * rows;
    const int64_t r1 = r0 + rows < n ? r0 + rows : n;
    const bool kin = 4 * lrow < K, min_ = 4 * lrow < M;
    float *g = sG[wave];

    f32x4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);

    // the 16 rows from `r` on, as the transposed product wants them; rows past the block's range read as zero
    auto fetch = [&](int64_t r, float4(&pa)[4], float4(&q)[4], float4(&y)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t row = r + 4 * u + lk;
            const bool rv = row < r1;
            pa[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            q[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            y[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rv && kin) pa[u] = *reinterpret_cast<const float4 *>(P + (size_t)row * K + 4 * lrow);
            if (rv && min_) {
                q[u] = *reinterpret_cast<const float4 *>(dY + (size_t)row * M + 4 * lrow);
                if (MASK) y[u] = *reinterpret_cast<const float4 *>(Y + (size_t)row * M + 4 * lrow);
            }
        }
    };

    float4 pa[4], q[4], y[4];
    int64_t r = r0 + 16 * wave;
    if (r < r1) fetch(r, pa, q, y);
    for (; r < r1; r += 16 * kBfWaves) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (MASK) {
                q[u].x = y[u].x > 0.0f ? q[u].x : 0.0f;
                q[u].y = y[u].y > 0.0f ? q[u].y : 0.0f;
                q[u].z = y[u].z > 0.0f ? q[u].z : 0.0f;
                q[u].w = y[u].w > 0.0f ? q[u].w : 0.0f;
            }
            if (WANT_R) *reinterpret_cast<float4 *>(g + (4 * u + lk) * kBfLd + 4 * lrow) = q[u];
            bsum.x += q[u].x;
            bsum.y += q[u].y;
            bsum.z += q[u].z;
            bsum.w += q[u].w;
        }
        // the next 16 rows travel while this turn's 128 MFMAs run
        float4 pa_n[4], q_n[4], y_n[4];
        fetch(r + 16 * kBfWaves, pa_n, q_n, y_n);
        // dW += P^T G: the reduction index of the MFMA is the row
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float av[4] = {pa[u].x, pa[u].y, pa[u].z, pa[u].w}, bv[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
        if (WANT_R) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // R^T = W G^T: the lane's reduction indices are m = 16*lk + s, s = 0..15, on both operands
            float gb[16];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float4 v = *reinterpret_cast<const float4 *>(g + lrow * kBfLd + 16 * lk + 4 * c);
                gb[4 * c] = v.x;
                gb[4 * c + 1] = v.y;
                gb[4 * c + 2] = v.z;
                gb[4 * c + 3] = v.w;
            }
            f32x4 d[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) d[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float4 w4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    w4[t] = *reinterpret_cast<const float4 *>(sW + (16 * t + lrow) * kBfLd + 16 * lk + 4 * c);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(w4[t].x, gb[4 * c], d[t], 0, 0, 0);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(w4[t].y, gb[4 * c + 1], d[t], 0, 0, 0);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(w4[t].z, gb[4 * c + 2], d[t], 0, 0, 0);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(w4[t].w, gb[4 * c + 3], d[t], 0, 0, 0);
            }
            // MFMA result row 4*lk + i of tile t is column 16*t + 4*lk + i of R, result column lrow is the row r + lrow
            const int64_t orow = r + lrow;
            if (orow < r1) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (16 * t + 4 * lk < K)
                        *reinterpret_cast<float4 *>(R + (size_t)orow * K + 16 * t + 4 * lk) =
                            make_float4(d[t][0], d[t][1], d[t][2], d[t][3]);
            }
            __builtin_amdgcn_wave_barrier();  // the tile is rewritten in the next turn
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            pa[u] = pa_n[u];
            q[u] = q_n[u];
            y[u] = y_n[u];
        }
    }

    const size_t slot = (size_t)blockIdx.x * kBfWaves + wave;
    float *mine = part_w + slot * (size_t)K * M;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = 4 * (4 * lk + i) + a, m = 4 * lrow + b;
                if (k < K && m < M) mine[(size_t)k * M + m] = acc[a][b][i];
            }
    if (part_b) {
        // the four lanes lrow, lrow + 16, .. hold the sums over the rows 4u + lk of the same four columns
        bsum.x += __shfl_xor(bsum.x, 16);
        bsum.y += __shfl_xor(bsum.y, 16);
        bsum.z += __shfl_xor(bsum.z, 16);
        bsum.w += __shfl_xor(bsum.w, 16);
        bsum.x += __shfl_xor(bsum.x, 32);
        bsum.y += __shfl_xor(bsum.y, 32);
        bsum.z += __shfl_xor(bsum.z, 32);
        bsum.w += __shfl_xor(bsum.w, 32);
        if (lk == 0 && min_) *reinterpret_cast<float4 *>(part_b + slot * (size_t)M + 4 * lrow) = bsum;
    }
}

// Sum of `count` partial arrays (a multiple of 32) in two levels, both with coalesced reads; the 32 sums of
// the first level go behind the partial arrays.
static void reduce_all(int count, int64_t len, float *partials, float *C, hipStream_t s)
{
    float *mid = partials + (size_t)count * len;
    const unsigned bx = (unsigned)((len + 255) / 256);
    hipLaunchKernelGGL(k_reduce_partials, dim3(bx, kRedGroups), dim3(256), 0, s, count / kRedGroups, len, partials, mid);
    hipLaunchKernelGGL(k_reduce_partials, dim3(bx, 1), dim3(256), 0, s, kRedGroups, len, mid, C);
}

// Shapes the one-pass kernel covers: below 33 columns most of its MFMA work would be padding.
static bool bwd_fused_shape(int32_t K, int32_t M)
{
    return K % 4 == 0 && M % 4 == 0 && K > 32 && K <= 64 && M > 32 && M <= 64;
}

// dW = P^T G, db = column sums of G (if wanted), R = G W^T (if wanted) with G = dY masked by Y > 0 (if Y) in one pass.
static int bwd_update_fused(int32_t n, int32_t K, int32_t M, const float *P, const float *dY, const float *Y,
                            const float *W, float *R, float *dW, float *db, float *partials, hipStream_t s)
{
    float *part_w = partials;
    float *part_b = db ? partials + (size_t)(kBfPartials + kRedGroups) * K * M : nullptr;
    const dim3 grid(kBfBlocks), block(64 * kBfWaves);
    if (Y && R) hipLaunchKernelGGL((k_bwd_update_fused<true, true>), grid, block, 0, s, n, K, M, P, dY, Y, W, R, part_w, part_b);
    else if (Y) hipLaunchKernelGGL((k_bwd_update_fused<true, false>), grid, block, 0, s, n, K, M, P, dY, Y, W, R, part_w, part_b);
    else if (R) hipLaunchKernelGGL((k_bwd_update_fused<false, true>), grid, block, 0, s, n, K, M, P, dY, Y, W, R, part_w, part_b);
    else hipLaunchKernelGGL((k_bwd_update_fused<false, false>), grid, block, 0, s, n, K, M, P, dY, Y, W, R, part_w, part_b);
    reduce_all(kBfPartials, (int64_t)K * M, part_w, dW, s);
    if (db) reduce_all(kBfPartials, (int64_t)M, part_b, db, s);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

static int gemm_tn(int32_t n, int32_t K, int32_t M, const float *P, const float *Q, float *C, float *partials,
                   hipStream_t s)
{
    const dim3 block(64 * kTnWaves);
    // the 16-byte form spreads 64 columns over a lane group's 16 accumulator tiles: with 32 columns or fewer on
    // either side half of its MFMAs and more are padding, and the 4-byte form is the faster one (measured)
    const bool v4 = K > 32 && M > 32 && K % 4 == 0 && M % 4 == 0 && ((uintptr_t)P | (uintptr_t)Q) % 16 == 0;
    if (v4) {
        const int kgroups = (K + 63) / 64, mgroups = (M + 63) / 64;
        hipLaunchKernelGGL(k_gemm_tn_partial_v4, dim3(kTnBlocks, (unsigned)(kgroups * mgroups)), block, 0, s, n, K, M, P, Q,
                           partials, mgroups);
    } else {
        // tiles per wave: up to 4 x up to 4 (16 accumulators of 4 registers)
        const int ktiles = (K + 15) / 16, mtiles = (M + 15) / 16;
        const int MT = mtiles >= 4 ? 4 : (mtiles >= 2 ? 2 : 1);
        const int KT = ktiles >= 3 ? 4 : (ktiles == 2 ? 2 : 1);
        const int kgroups = (ktiles + KT - 1) / KT, mgroups = (mtiles + MT - 1) / MT;
        const dim3 grid(kTnBlocks, (unsigned)(kgroups * mgroups));
#define GNN_TN_CASE(kt, mt) \
    if (KT == kt && MT == mt) hipLaunchKernelGGL((k_gemm_tn_partial<kt, mt>), grid, block, 0, s, n, K, M, P, Q, partials, mgroups)
        GNN_TN_CASE(4, 4); GNN_TN_CASE(4, 2); GNN_TN_CASE(4, 1);
        GNN_TN_CASE(2, 4); GNN_TN_CASE(2, 2); GNN_TN_CASE(2, 1);
        GNN_TN_CASE(1, 4); GNN_TN_CASE(1, 2); GNN_TN_CASE(1, 1);
#undef GNN_TN_CASE
    }
    reduce_all(kTnPartials, (int64_t)K * M, partials, C, s);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

struct BwdLayout {
    size_t base;      // partition of the transposed graph (ws_layout without intermediate)
    size_t dz;        // float[n*out_dim]
    size_t dh;        // float[n*max(in_dim,out_dim)]
    size_t wt;        // float[in_dim*out_dim]
    size_t partials;  // partial dW (and db) of every wave, and the first level of their sums
    size_t total;
};

static BwdLayout bwd_layout(int32_t n, int64_t nnz, int32_t in_dim, int32_t out_dim, int32_t ngs)
{
    BwdLayout B;
    B.base = 0;
    size_t off = ws_layout(n, nnz, 0, ngs).total;
    const int32_t mx = in_dim > out_dim ? in_dim : out_dim;
    B.dz = off;
    off += align_up(sizeof(float) * (size_t)n * out_dim);
    B.dh = off;
    off += align_up(sizeof(float) * (size_t)n * mx);
    B.wt = off;
    off += align_up(sizeof(float) * (size_t)in_dim * out_dim);
    B.partials = off;
    size_t pb = sizeof(float) * (size_t)(kTnPartials + kRedGroups) * in_dim * out_dim;
    const size_t bb = sizeof(float) * (size_t)(kColsumBlocks + kRedGroups) * out_dim;
    if (pb < bb) pb = bb;
    if (bwd_fused_shape(in_dim, out_dim))  // partial dW and db of every wave of the one-pass kernel
        pb = sizeof(float) * (size_t)(kBfPartials + kRedGroups) * ((size_t)in_dim * out_dim + out_dim);
    off += align_up(pb);
    B.total = off;
    return B;
}

}  // namespace gnn

using namespace gnn;

extern "C" {

size_t gnn_backward_workspace_bytes(int32_t n, int64_t nnz, int32_t in_dim, int32_t out_dim, int32_t ngs)
{
    if (n < 0 || nnz < 0 || in_dim <= 0 || out_dim <= 0 || ngs < 0) return 0;
    // capacity for whatever group size the model may pick when ngs == 0 (ngs = 1 is the upper bound)
    const int32_t cap_ngs = ngs > 0 ? ngs : 1;
    return bwd_layout(n, nnz, in_dim, out_dim, cap_ngs).total +
           part_rows_bytes(ng_upper_bound(n, nnz, cap_ngs), kPartMinTile, in_dim > out_dim ? in_dim : out_dim);
}

int gnn_layer_backward(int kind, int32_t n, int64_t nnz, const int32_t *rowptr_t, const int32_t *colidx_t,
                       const float *ew_t, float eps, const float *P, int32_t in_dim, const float *W, int32_t out_dim,
                       int relu, const float *Y, const float *dY, float *dX, float *dW, float *db, int32_t ngs,
                       int32_t dw, int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    if (kind != GNN_GCN && kind != GNN_GIN) return GNN_EINVAL;
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31) || in_dim <= 0 || out_dim <= 0 || ngs < 0) return GNN_EINVAL;
    if (n == 0) return GNN_OK;
    if (!P || !W || !dY || !dW || (relu && !Y)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int32_t agg_dim = kind == GNN_GCN ? out_dim : in_dim;
    int32_t ngs_r = ngs, dw_r = dw, wpb_r = waves_per_block;
    decide_defaults(n, nnz, 0, agg_dim, 1, &ngs_r, &dw_r, &wpb_r);  // only ngs matters here: it fixes the layout
    const BwdLayout B = bwd_layout(n, nnz, in_dim, out_dim, ngs_r);
    if (!workspace || ((uintptr_t)workspace) % kAlign != 0 || workspace_bytes < B.total) return GNN_EWORKSPACE;
    char *ws = (char *)workspace;
    float *dZbuf = (float *)(ws + B.dz), *dHbuf = (float *)(ws + B.dh), *Wt = (float *)(ws + B.wt);
    float *partials = (float *)(ws + B.partials);
    const int64_t total = (int64_t)n * out_dim;

    const bool aligned16 = (((uintptr_t)P | (uintptr_t)dY | (uintptr_t)Y | (uintptr_t)W | (uintptr_t)dX) % 16) == 0;
    const bool one_pass = aligned16 && bwd_fused_shape(in_dim, out_dim);
    if (kind == GNN_GIN && one_pass) {
        // dW, db and dA = G W^T in one pass over the rows (G is not stored), then the aggregation of dA
        int rc = bwd_update_fused(n, in_dim, out_dim, P, dY, relu ? Y : nullptr, W, dX ? dHbuf : nullptr, dW, db, partials, s);
        if (rc != GNN_OK || !dX) return rc;
        return aggregate_impl(true, 1.0f + eps, n, nnz, rowptr_t, colidx_t, nullptr, dHbuf, dX, in_dim, ngs_r, dw,
                              waves_per_block, flags, nullptr, 0, workspace, workspace_bytes, B.total, s, nullptr, nullptr,
                              nullptr);
    }

    // through the activation
    const float *dZ = dY;
    if (relu) {
        int64_t blocks = (total + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(k_relu_mask, dim3((unsigned)blocks), dim3(256), 0, s, total, dY, Y, dZbuf);
        dZ = dZbuf;
    }
    if (db) {
        hipLaunchKernelGGL(k_colsum_partial, dim3(kColsumBlocks), dim3(256), 0, s, n, out_dim, dZ, partials);
        reduce_all(kColsumBlocks, (int64_t)out_dim, partials, db, s);
    }
    hipLaunchKernelGGL(k_transpose, dim3((unsigned)((in_dim * out_dim + 255) / 256)), dim3(256), 0, s, in_dim, out_dim, W,
                       Wt);
    GNN_HIP_TRY(hipGetLastError());

    if (kind == GNN_GCN) {
        // forward: Y = act(A_hat (X W) + b), P = X.  dH = A_hat^T dZ, dW = X^T dH, dX = dH W^T
        int rc = aggregate_impl(false, 0.0f, n, nnz, rowptr_t, colidx_t, ew_t, dZ, dHbuf, out_dim, ngs_r, dw,
                                waves_per_block, flags, nullptr, 0, workspace, workspace_bytes, B.total, s, nullptr, nullptr,
                                nullptr);
        if (rc != GNN_OK) return rc;
        if (one_pass && dX) return bwd_update_fused(n, in_dim, out_dim, P, dHbuf, nullptr, W, dX, dW, nullptr, partials, s);
        rc = gemm_tn(n, in_dim, out_dim, P, dHbuf, dW, partials, s);
        if (rc != GNN_OK) return rc;
        if (dX) return update_gemm_impl(n, out_dim, in_dim, dHbuf, Wt, nullptr, 0, dX, s);
        return GNN_OK;
    }
    // GIN forward: Y = act(A W + b) with A = (1+eps) X + sum_N X, P = A.
    // dW = A^T dZ, dA = dZ W^T, dX = (1+eps) dA + sum over the transposed graph of dA
    int rc = gemm_tn(n, in_dim, out_dim, P, dZ, dW, partials, s);
    if (rc != GNN_OK) return rc;
    if (!dX) return GNN_OK;
    rc = update_gemm_impl(n, out_dim, in_dim, dZ, Wt, nullptr, 0, dHbuf, s);
    if (rc != GNN_OK) return rc;
    return aggregate_impl(true, 1.0f + eps, n, nnz, rowptr_t, colidx_t, nullptr, dHbuf, dX, in_dim, ngs_r, dw,
                          waves_per_block, flags, nullptr, 0, workspace, workspace_bytes, B.total, s, nullptr, nullptr,
                          nullptr);
}

}  // extern "C"
