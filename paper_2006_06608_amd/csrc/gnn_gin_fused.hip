// GIN layer with the Update fused into the Aggregation (an MI355X addition; the paper runs the two
// phases as separate kernels): out = act(((1+eps) X + sum_N X) W + b) in one pass.
//
// The persistent, software-pipelined aggregation (see gnn_aggregate_pipe.hip) leaves every target
// node of a tile as one row of an LDS tile A[T][K] (Algorithm 1 slots, now used for all nodes).
// After the tile's single barrier the block multiplies A by W with v_mfma_f32_16x16x4_f32 -- each
// wave owns 16 output columns whose W fragments stay in registers for the whole kernel -- and
// writes act(. + b) for nodes complete in the tile.  A node that spans tiles contributes
// (partial row) W with global atomic adds, which is valid because the product is linear; its bias
// and activation are applied by the follow-up kernel that already serves such rows.  The
// aggregated matrix never goes to HBM and the separate GEMM kernel disappears.
//
// Opt-in (GNN_FLAG_FUSION).  Measured on the R-MAT configuration (1,048,576 nodes, Dim 64 -> 64) the
// fused layer takes 690 us against 597 us for aggregation + GEMM run separately: all rows pass
// through LDS, the register budget of the W fragments lowers occupancy to 4 waves per SIMD, the MFMA
// phase sits on every tile's critical path, and the 48 % of rows without neighbours need the
// product anyway.  It is kept for shapes where the aggregated matrix dominates the traffic.
//
// LDS slots are triple-buffered: the buffer read by the MFMA phase of tile i is cleared after the
// barrier of tile i+1 and refilled during tile i+3, so one barrier per tile still suffices.
#include <hip/hip_runtime.h>

#include "gnn_launch.h"
#include "gnn_pipe_common.h"

namespace gnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct FusedParams {
    AggParams a;     // X = layer input [n,K], dim = K, self_scale = 1 + eps; out/bias/relu unused
    const float *W;  // [K,M]
    const float *b;  // [M] or null
    float *out;      // [n,M]
    int M;
    int relu;
    int ct;          // 16-column tiles of the output
};

// C[16 x 16] = A_tile[16 x 16*NS] . W fragment, for one row tile.
template <int NS>
__device__ __forceinline__ f32x4 tile_mfma(const float *arow, const float (&wreg)[4 * NS], int lk)
{
    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const float4 a4 = *reinterpret_cast<const float4 *>(arow + 16 * s + 4 * lk);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, wreg[4 * s + 0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, wreg[4 * s + 1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, wreg[4 * s + 2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, wreg[4 * s + 3], acc, 0, 0, 0);
    }
    return acc;
}

template <int ITER, int U, int NS>
__global__ __launch_bounds__(256) void k_gin_layer_fused(FusedParams fp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const AggParams &p = fp.a;
    const WsHeader *hdr = p.hdr;
    if (!header_ok(hdr, p)) return;

    constexpr int VEC = 4;
    constexpr int KP = 16 * NS;   // K padded to the MFMA step group
    constexpr int LDA = KP + 4;   // row stride of the LDS tile (bank spread for the 16-byte reads)
    const int T = p.T, dim = p.dim, ngs = p.ngs, M = fp.M;
    const int64_t num_ng = hdr->num_ng;
    const int64_t tiles = (num_ng + T - 1) / T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int dwl_log2 = p.dwl_log2, dwl = 1 << dwl_log2;
    const int G = 64 >> dwl_log2;
    const int tlane = lane & (dwl - 1);
    const int team_in_wave = lane >> dwl_log2;
    const int wcap = G * ngs;
    const int lrow = lane & 15, lk = lane >> 4;

    // LDS: [3][T][LDA] tile | [3][T] node of slot | [3][T] flags of slot | [2][nwaves][wcap] indices | [64] list
    float *s_A = reinterpret_cast<float *>(smem);
    int *s_node = reinterpret_cast<int *>(s_A + 3 * (size_t)T * LDA);
    int *s_flag = s_node + 3 * T;
    int *s_col = s_flag + 3 * T;
    int *s_list = s_col + 2 * (size_t)nwaves * wcap;

    for (int i = tid; i < 3 * T * LDA; i += blockDim.x) s_A[i] = 0.0f;
    for (int i = tid; i < 3 * T; i += blockDim.x) s_flag[i] = 0;

    // this wave's output columns and its W fragments: wreg[4s+q] = W[16s + 4*lk + q][16*ct_w + lrow]
    const int ct_w = wave % fp.ct;
    const int rt_first = wave / fp.ct, rt_step = nwaves / fp.ct;  // row tiles handled by this wave
    const int col = 16 * ct_w + lrow;
    float wreg[4 * NS];
#pragma unroll
    for (int j = 0; j < 4 * NS; ++j) {
        const int k = 16 * (j >> 2) + 4 * lk + (j & 3);
        wreg[j] = (k < dim && col < M) ? fp.W[(size_t)k * M + col] : 0.0f;
    }
    const float bcol = (fp.b && col < M) ? fp.b[col] : 0.0f;
    __syncthreads();

    const int64_t B = gridDim.x, b = blockIdx.x;
    const bool remap = p.xcd_remap && (B % kNumXcd == 0);
    const int64_t J = B / kNumXcd, xj = b / kNumXcd, xx = b % kNumXcd;
    auto tile_of = [&](int64_t i) -> int64_t { return remap ? (i * kNumXcd + xx) * J + xj : i * B + b; };
    auto fetch_tuples = [&](int64_t tile) -> NgEntry {
        NgEntry e;
        e.node = -1;
        e.start = e.end = e.flags = 0;
        if (tile < tiles) {
            const int64_t g = tile * T + lane;
            if (lane < T && g < num_ng) e = p.ng[g];
        }
        return e;
    };
    int cpre[kPipeIdxLoads];
    auto prefetch_idx = [&](const TileView &V) {
#pragma unroll
        for (int r = 0; r < kPipeIdxLoads; ++r) {
            const int k = lane + 64 * r;
            cpre[r] = 0;
            if (k < V.ws1 - V.ws0) cpre[r] = load_stream(&p.colidx[V.ws0 + k]);
        }
    };
    auto commit_idx = [&](const TileView &V, int buf) {
        int *dc = s_col + ((size_t)buf * nwaves + wave) * wcap;
#pragma unroll
        for (int r = 0; r < kPipeIdxLoads; ++r) {
            const int k = lane + 64 * r;
            if (k < V.ws1 - V.ws0) dc[k] = cpre[r];
        }
    };

    // Multiply the rows [0, nrows) of tile buffer `sb` by W and write them; every wave takes part.
    auto multiply_and_store = [&](int sb, int nrows) {
        const float *At = s_A + (size_t)sb * T * LDA;
        const int *nodes = s_node + sb * T, *flags = s_flag + sb * T;
        for (int rt = rt_first; rt * 16 < nrows; rt += rt_step) {
            const f32x4 acc = tile_mfma<NS>(At + (size_t)(16 * rt + lrow) * LDA, wreg, lk);
            if (col < M) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 16 * rt + 4 * lk + i;  // MFMA result row -> slot
                    if (r < nrows) {
                        const int node = nodes[r];
                        float *o = fp.out + (size_t)node * M + col;
                        if ((flags[r] & 3) == 3) {
                            float v = acc[i] + bcol;
                            if (fp.relu) v = fmaxf(v, 0.0f);
                            *o = v;
                        } else {
                            atomicAdd(o, acc[i]);
                        }
                    }
                }
            }
        }
    };
    // Clear tile buffer `sb` (rows [0, nrows)) for its next use; every thread takes part.
    auto clear_tile = [&](int sb, int nrows) {
        float *At = s_A + (size_t)sb * T * LDA;
        for (int i = tid; i < nrows * LDA; i += blockDim.x) At[i] = 0.0f;
        for (int i = tid; i < nrows; i += blockDim.x) s_flag[sb * T + i] = 0;
    };

    NgEntry tl_next = fetch_tuples(tile_of(1));
    TileView cur = derive_tile(fetch_tuples(tile_of(0)), dwl_log2, T);
    prefetch_idx(cur);
    commit_idx(cur, 0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    int prev_rows = 0;  // slots used by the previous tile (to be cleared after this tile's barrier)
    int64_t it = 0;
    for (;; ++it) {
        if (tile_of(it) >= tiles) break;
        const int buf = (int)(it & 1), sb = (int)(it % 3), sb_prev = (int)((it + 2) % 3);
        const NgEntry tl_after = fetch_tuples(tile_of(it + 2));
        const TileView nxt = derive_tile(tl_next, dwl_log2, T);
        prefetch_idx(nxt);

        const NgEntry e = cur.e;
        const int len = cur.valid ? e.end - e.start : 0;
        const int off = e.start - cur.ws0;
        const bool first = (e.flags & 1) != 0;
        const int *lc = s_col + ((size_t)buf * nwaves + wave) * wcap + off;
        float *At = s_A + (size_t)sb * T * LDA;

        const unsigned long long cont = __ballot(cur.valid && !cur.leader && team_in_wave > 0);
        const bool seg_head = cur.valid && (team_in_wave == 0 || cur.leader);
        int lastflag = cur.valid ? (e.flags & 2) : 0;
        bool lastflag_done = false;

        for (int c0 = 0; c0 < p.iter_total; c0 += ITER) {
            float acc[ITER][VEC];
            bool dok[ITER];
#pragma unroll
            for (int c = 0; c < ITER; ++c) {
                dok[c] = ((c0 + c) * dwl + tlane) * VEC < dim;
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[c][j] = 0.0f;
            }
            const float *xb = p.X + (size_t)(c0 * dwl + tlane) * VEC;
            for (int base = 0; base < len; base += U) {
                int colv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) colv[u] = (base + u < len) ? lc[base + u] : -1;
                float v[U][ITER][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        if (colv[u] >= 0 && dok[c]) {
                            load_vec<VEC>(v[u][c], xb + (size_t)colv[u] * dim + (size_t)c * dwl * VEC);
                        } else {
#pragma unroll
                            for (int j = 0; j < VEC; ++j) v[u][c][j] = 0.0f;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int c = 0; c < ITER; ++c)
#pragma unroll
                        for (int j = 0; j < VEC; ++j) acc[c][j] += v[u][c][j];
            }
            if (cont != 0ull) {
                const int key = cur.valid ? e.node : -1;
                for (int o = dwl; o < 64; o <<= 1) {
                    const int okey = __shfl_down(key, o);
                    const bool take = (lane + o < 64) && key >= 0 && okey == key;
#pragma unroll
                    for (int c = 0; c < ITER; ++c)
#pragma unroll
                        for (int j = 0; j < VEC; ++j) {
                            const float ov = __shfl_down(acc[c][j], o);
                            if (take) acc[c][j] += ov;
                        }
                    if (!lastflag_done) {
                        const int ol = __shfl_down(lastflag, o);
                        if (take) lastflag |= ol;
                    }
                }
            }
            lastflag_done = true;
            if (seg_head) {
                float *srow = At + (size_t)cur.slot * LDA;
#pragma unroll
                for (int c = 0; c < ITER; ++c) {
                    const int d = ((c0 + c) * dwl + tlane) * VEC;
                    if (d < dim) {
                        if (first) {  // the team holding the node's first group also brings the self term
                            float xs[VEC];
                            load_vec<VEC>(xs, p.X + (size_t)e.node * dim + d);
#pragma unroll
                            for (int j = 0; j < VEC; ++j) acc[c][j] = fmaf(p.self_scale, xs[j], acc[c][j]);
                        }
#pragma unroll
                        for (int j = 0; j < VEC; ++j) atomicAdd(&srow[d + j], acc[c][j]);
                    }
                }
            }
        }
        if (seg_head && tlane == 0) {
            if (cur.leader) s_node[sb * T + cur.slot] = e.node;
            const int fl = (cur.leader && first ? 1 : 0) | (lastflag != 0 ? 2 : 0);
            if (fl) atomicOr(&s_flag[sb * T + cur.slot], fl);
        }
        __syncthreads();

        multiply_and_store(sb, cur.nslots);
        if (it > 0) clear_tile(sb_prev, prev_rows);  // everyone finished reading it before this barrier
        prev_rows = cur.nslots;

        commit_idx(nxt, buf ^ 1);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        cur = nxt;
        tl_next = tl_after;
    }

    // rows without any entry: out = act((1+eps) x W + b), sixteen-row tiles through the same MFMA path.
    // Buffers 0..2 are reused as one scratch tile of up to T rows (buffer 0), after a barrier.
    __syncthreads();
    clear_tile(0, T);
    clear_tile(1, T);
    clear_tile(2, T);
    __syncthreads();
    const int64_t nchunks = ((int64_t)p.n + 63) / 64;
    const int nteams = nwaves * G, team = wave * G + team_in_wave;
    for (int64_t c = b; c < nchunks; c += B) {
        // wave 0 lists the empty nodes of this 64-node chunk
        if (wave == 0) {
            const int64_t v = c * 64 + lane;
            const bool empty = v < p.n && p.ngptr[v] == p.ngptr[v + 1];
            const unsigned long long m = __ballot(empty);
            if (empty) s_list[1 + __popcll(m & ((1ull << lane) - 1ull))] = lane;
            if (lane == 0) s_list[0] = __popcll(m);
        }
        __syncthreads();
        const int cnt = s_list[0];
        for (int base = 0; base < cnt; base += T) {
            const int rows = cnt - base < T ? cnt - base : T;
            for (int r = team; r < rows; r += nteams) {
                const int64_t node = c * 64 + s_list[1 + base + r];
                for (int cc = 0; cc < p.iter_total; ++cc) {
                    const int d = (cc * dwl + tlane) * VEC;
                    if (d >= dim) break;
                    float xs[VEC];
                    load_vec<VEC>(xs, p.X + (size_t)node * dim + d);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) s_A[(size_t)r * LDA + d + j] = p.self_scale * xs[j];
                }
                if (tlane == 0) {
                    s_node[r] = (int)node;
                    s_flag[r] = 3;
                }
            }
            __syncthreads();
            multiply_and_store(0, rows);
            __syncthreads();
        }
        __syncthreads();
    }
}

template <int ITER, int U>
static const void *fused_fn2(int ns)
{
    switch (ns) {
        case 1: return (const void *)k_gin_layer_fused<ITER, U, 1>;
        case 2: return (const void *)k_gin_layer_fused<ITER, U, 2>;
        case 4: return (const void *)k_gin_layer_fused<ITER, U, 4>;
        default: return (const void *)k_gin_layer_fused<ITER, U, 8>;
    }
}

static const void *fused_fn(int iter, int ns)
{
    switch (iter) {
        case 1: return fused_fn2<1, 8>(ns);
        case 2: return fused_fn2<2, 4>(ns);
        case 3: return fused_fn2<3, 4>(ns);
        default: return fused_fn2<4, 2>(ns);
    }
}

// Step groups (of 16) to which K is padded, or 0 if the fused kernel does not cover this shape.
static int fused_ns(int K)
{
    if (K <= 16) return 1;
    if (K <= 32) return 2;
    if (K <= 64) return 4;
    if (K <= 128) return 8;
    return 0;
}

// Tries the fused GIN layer.  Returns GNN_OK after enqueueing it, 1 if the shape or the launch
// shape is outside what it covers (the caller then runs aggregation and GEMM separately), < 0 on error.
int try_gin_layer_fused(AggParams &p, int vec, int wpb, const float *W, const float *b, float *out, int M, int relu,
                        int64_t tiles_upper, bool force, hipStream_t s)
{
    const int K = p.dim;
    const int ns = fused_ns(K);
    const int T = p.T, G = 64 >> p.dwl_log2;
    if (vec != 4 || ns == 0 || M > 64 || T > 64 || T % 16 != 0) return 1;
    if ((int64_t)G * p.ngs > 64 * kPipeIdxLoads) return 1;
    const int ct = (M + 15) / 16;
    if (wpb % ct != 0 || wpb > 4) return 1;  // the kernel is compiled for blocks of up to 4 waves
    if (p.iter_total > 4) return 1;
    if (((uintptr_t)W | (uintptr_t)out) % 4 != 0) return 1;
    const int lda = 16 * ns + 4;
    const size_t lds = (size_t)3 * T * lda * 4 + (size_t)6 * T * 4 + (size_t)2 * wpb * G * p.ngs * 4 + 65 * 4;
    if (lds > kMaxLdsBytes) return 1;
    const void *fn = fused_fn(p.iter_total, ns);
    int dev = 0, cus = 0, per_cu = 0;
    GNN_HIP_TRY(hipGetDevice(&dev));
    GNN_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    GNN_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, wpb * 64, lds));
    if (per_cu < 1) return 1;
    int64_t blocks = (int64_t)per_cu * cus;
    (void)force;
    if (blocks > tiles_upper) blocks = tiles_upper > 0 ? tiles_upper : 1;
    if (blocks >= kNumXcd) blocks = blocks / kNumXcd * kNumXcd;
    // rows of `out` that will receive atomic adds are zeroed first; rows without entries are written
    // by the fused kernel itself
    AggParams po = p;
    po.out = out;
    po.dim = M;
    po.bias = b;
    po.relu = relu;
    po.do_empty = 1;
    launch_agg_init(po, false, s);
    FusedParams fp;
    fp.a = p;
    fp.W = W;
    fp.b = b;
    fp.out = out;
    fp.M = M;
    fp.relu = relu;
    fp.ct = ct;
    void *args[] = {(void *)&fp};
    GNN_HIP_TRY(hipLaunchKernel(fn, dim3((unsigned)blocks), dim3((unsigned)(wpb * 64)), args, lds, s));
    if (b || relu) launch_agg_epilogue_spanning(po, s);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

}  // namespace gnn
