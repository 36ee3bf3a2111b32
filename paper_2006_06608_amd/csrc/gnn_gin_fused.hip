// GIN layer with the Update fused into the Aggregation, built on the general aggregation kernel:
// out = act(((1+eps) X + sum_N X) W + b) in one launch (an MI355X addition; the paper runs the two
// phases as separate kernels).
//
// A block aggregates its neighbor groups exactly as k_aggregate does, but every target node of the
// block ends up as one row of an LDS tile A[T][K] (the Algorithm 1 slots, the waves adding in wave
// order).  After the barrier the block multiplies the tile by W, which it staged in LDS at its start,
// with v_mfma_f32_16x16x4_f32: wave w owns the 16 output columns w mod ct of the row tiles
// w / ct, w / ct + W/ct, ...  A node complete in the block gets act(row W + b) stored.  For a node
// that spans blocks the product is applied to the block's partial row, which is valid because the
// product is linear: (sum of partial rows) W = sum of (partial row W); the transformed partial row
// (out_dim floats) then takes the ordered flush: device-coherent store, arrival counter, the block
// that arrives last adds the partial rows in block order and applies bias and activation.  Rows
// without any entry, act((1+eps) x W + b), are served by blocks appended to the grid whose waves
// compact 16 such rows at a time and feed them to the same MFMA path straight from global memory.
// The aggregated matrix never goes to HBM and the separate GEMM kernel disappears.
#include <hip/hip_runtime.h>

#include "gnn_launch.h"

namespace gnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct FusedParams {
    AggParams a;     // X = layer input [n,K], dim = K, self_scale = 1 + eps, part_rows [2*tiles][M], cnt
    const float *W;  // [K,M]
    const float *b;  // [M] or null
    float *out;      // [n,M]
    int M;
    int relu;
    int ct;          // 16-column tiles of the output (1..4)
    int a_rows;      // rows of the LDS tile: T rounded up to whole 16-row MFMA tiles
};

__device__ __forceinline__ float act_bias(float v, float bcol, int relu)
{
    v += bcol;
    return relu ? fmaxf(v, 0.0f) : v;
}

template <int ITER, int U, int NS>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(ITER == 1 ? 6 : 5)))
void k_gin_layer_fused(FusedParams fp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const AggParams &p = fp.a;
    const WsHeader *hdr = p.hdr;
    if (!header_ok(hdr, p)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) note_stale(p.hdr, p);
        return;
    }
    constexpr int VEC = 4;
    constexpr int KP = 16 * NS;  // K padded to whole MFMA step groups
    constexpr int LDA = KP + 4;  // row stride of the LDS tile
    const int T = p.T, dim = p.dim, M = fp.M, ct = fp.ct;
    const int LDW = 16 * ct + 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = blockDim.x >> 6;
    const int dwl_log2 = p.dwl_log2, dwl = 1 << dwl_log2;
    const int tlane = lane & (dwl - 1);
    const int team_in_wave = lane >> dwl_log2;
    const int lrow = lane & 15, lk = lane >> 4;

    // LDS: wave counts [16] | s_last [T] | s_node [T] | s_state [T] | s_col [T*ngs] | (16-byte aligned)
    //      s_W [KP][LDW] | s_A [a_rows][LDA] | per-wave lists [nw][64]
    int *s_wave_cnt = reinterpret_cast<int *>(smem);
    int *s_last = s_wave_cnt + kMaxWavesPerBlock;
    int *s_node = s_last + T;
    int *s_state = s_node + T;
    int *s_col = s_state + T;
    size_t off_w = (size_t)(kMaxWavesPerBlock + 3 * T + (size_t)T * p.ngs) * 4;
    off_w = (off_w + 15) & ~(size_t)15;
    float *s_W = reinterpret_cast<float *>(smem + off_w);
    float *s_A = s_W + (size_t)KP * LDW;
    int *s_list = reinterpret_cast<int *>(s_A + (size_t)fp.a_rows * LDA);

    // One tile per block (several per block measured slower: they run one after the other, and the
    // loop costs registers).  Surplus blocks of the over-sized grid leave before they touch anything.
    const bool tile_block = (int64_t)blockIdx.x < p.tile_blocks;
    const int64_t num_ng = hdr->num_ng;
    const int64_t tile = blockIdx.x;
    if (tile_block && tile * T >= num_ng) return;

    // W into LDS (zero padded to KP rows and 64 columns): thread t takes the float4 (t mod 16) of the
    // rows t/16, t/16 + blockDim/16, ...; the loads overlap with what follows
    {
        const int c = (tid & 15) * 4;
        const bool vecw = (M % 4 == 0) && (((uintptr_t)fp.W & 15) == 0);
        for (int k = tid >> 4; k < KP; k += blockDim.x >> 4) {
            float4 w4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < dim && c < M) {
                const float *src = fp.W + (size_t)k * M + c;
                if (vecw) {
                    w4 = *reinterpret_cast<const float4 *>(src);
                } else {
                    w4.x = src[0];
                    if (c + 1 < M) w4.y = src[1];
                    if (c + 2 < M) w4.z = src[2];
                    if (c + 3 < M) w4.w = src[3];
                }
            }
            if (c < 16 * ct) *reinterpret_cast<float4 *>(s_W + k * LDW + c) = w4;
        }
    }

    // this wave's output columns
    const int ct_w = wave % ct;
    const int rt_first = wave / ct, rt_step = nw / ct;
    const int col = 16 * ct_w + lrow;
    const float bcol = (fp.b && col < M) ? fp.b[col] : 0.0f;
    const float *wcol = s_W + 16 * ct_w + lrow;  // + k * LDW

    if (!tile_block) {
        // ---- rows without entries: act((1+eps) x W + b); every wave works alone
        __syncthreads();  // W is in LDS
        int *mylist = s_list + wave * 64;
        const int64_t nchunks = ((int64_t)p.n + 63) / 64;
        const int64_t first_chunk = ((int64_t)blockIdx.x - p.tile_blocks) * nw + wave;
        const int64_t chunk_stride = (int64_t)p.extra_blocks * nw;
        for (int64_t c = first_chunk; c < nchunks; c += chunk_stride) {
            const int64_t v = c * 64 + lane;
            const bool empty = v < p.n && p.ngptr[v] == p.ngptr[v + 1];
            const unsigned long long m = __ballot(empty);
            if (m == 0ull) continue;
            const int cnt = __popcll(m);
            if (empty) mylist[__popcll(m & ((1ull << lane) - 1ull))] = lane;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int base = 0; base < cnt; base += 16) {
                // lane (lrow, lk) feeds row `lrow` of this group of 16 rows, k = 16s + 4*lk .. +3
                const bool rok = base + lrow < cnt;
                const int64_t node = c * 64 + (rok ? mylist[base + lrow] : 0);
                float4 a4[NS];
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const int k = 16 * s + 4 * lk;
                    a4[s] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (rok && k < dim) a4[s] = *reinterpret_cast<const float4 *>(p.X + (size_t)node * dim + k);
                }
                for (int t = 0; t < ct; ++t) {
                    const float *wc = s_W + 16 * t + lrow;
                    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        const int k = 16 * s + 4 * lk;
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s].x, wc[(k + 0) * LDW], acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s].y, wc[(k + 1) * LDW], acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s].z, wc[(k + 2) * LDW], acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s].w, wc[(k + 3) * LDW], acc, 0, 0, 0);
                    }
                    const int cc = 16 * t + lrow;
                    const float bc = (fp.b && cc < M) ? fp.b[cc] : 0.0f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = base + 4 * lk + i;  // result row -> position in the list
                        if (r < cnt && cc < M) {
                            const int64_t nd = c * 64 + mylist[r];
                            fp.out[(size_t)nd * M + cc] = act_bias(p.self_scale * acc[i], bc, fp.relu);
                        }
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }

    int *s_shared = s_wave_cnt + kMaxWavesPerBlock - 1;  // 1: some node of the tile is shared by several waves
    {
        const int64_t g0 = tile * T;
        const BlockLayout lay = block_layout(p.ng, g0, num_ng, dwl_log2, s_wave_cnt);
        const NgEntry e = lay.e;

        // stage the tile's contiguous CSR range, clear the LDS tile
        const int64_t g_last = (g0 + T < num_ng ? g0 + T : num_ng) - 1;
        const int e0 = p.ng[g0].start;
        const int e1 = p.ng[g_last].end;
        for (int i = tid; i < e1 - e0; i += blockDim.x) s_col[i] = load_stream(&p.colidx[e0 + i]);
        for (int i = tid; i < T * LDA; i += blockDim.x) s_A[i] = 0.0f;
        for (int i = tid; i < T; i += blockDim.x) {
            s_last[i] = 0;
            s_state[i] = 0;
        }
        if (tid == 0) *s_shared = 0;
        __syncthreads();  // (this also publishes W)
        const int slot = block_layout_slot(lay, dwl_log2, s_wave_cnt);
        int nslots = 0;
        for (int w = 0; w < nw; ++w) nslots += s_wave_cnt[w];

        const int len = lay.valid ? e.end - e.start : 0;
        const int off = lay.valid ? e.start - e0 : 0;
        const bool first = (e.flags & 1) != 0;
        const unsigned long long cont = __ballot(lay.valid && !lay.leader && team_in_wave > 0);
        const bool seg_head = lay.valid && (team_in_wave == 0 || lay.leader);
        int lastflag = lay.valid ? (e.flags & 2) : 0;
        bool lastflag_done = false;

        for (int c0 = 0; c0 < p.iter_total; c0 += ITER) {
            float acc[ITER][VEC];
            bool dok[ITER];
            const float *xb = p.X + (size_t)(c0 * dwl + tlane) * VEC;
#pragma unroll
            for (int c = 0; c < ITER; ++c) {
                dok[c] = ((c0 + c) * dwl + tlane) * VEC < dim;
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[c][j] = 0.0f;
                if (first && len > 0 && dok[c]) {  // the node's own row, as one more term of its first group
                    float xs[VEC];
                    load_vec<VEC>(xs, xb + (size_t)e.node * dim + (size_t)c * dwl * VEC);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) acc[c][j] = p.self_scale * xs[j];
                }
            }
            for (int base = 0; base < len; base += U) {
                int colv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int cu = s_col[off + base + u];
                    colv[u] = base + u < len ? cu : -1;
                }
                float v[U][ITER][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        if (colv[u] >= 0 && dok[c]) {
                            load_vec<VEC>(v[u][c],
                                          xb + (size_t)(unsigned)colv[u] * (unsigned)dim + (size_t)c * dwl * VEC);
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
                const int key = lay.valid ? e.node : -1;
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
            // A node whose groups all sit in this wave owns its row of the tile: plain store.  Rows
            // shared by several waves are added wave after wave (the segment heads of one wave have
            // distinct target nodes), only in tiles that have such rows.
            const bool own_row = seg_head && first && lastflag != 0;
            if (seg_head) {
                if (own_row) {
                    float *srow = s_A + (size_t)slot * LDA;
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        const int d = ((c0 + c) * dwl + tlane) * VEC;
                        if (d < dim)
                            *reinterpret_cast<float4 *>(srow + d) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
                    }
                    if (tlane == 0) s_last[slot] = 1;
                } else if (tlane == 0) {
                    *s_shared = 1;
                }
            }
            __syncthreads();
            if (*s_shared != 0) {
                for (int w = 0; w < nw; ++w) {
                    if (wave == w && seg_head && !own_row) {
                        float *srow = s_A + (size_t)slot * LDA;
#pragma unroll
                        for (int c = 0; c < ITER; ++c) {
                            const int d = ((c0 + c) * dwl + tlane) * VEC;
                            if (d < dim) {
                                float4 cur = *reinterpret_cast<float4 *>(srow + d);
                                cur.x += acc[c][0];
                                cur.y += acc[c][1];
                                cur.z += acc[c][2];
                                cur.w += acc[c][3];
                                *reinterpret_cast<float4 *>(srow + d) = cur;
                            }
                        }
                        if (lastflag != 0 && tlane == 0) s_last[slot] = 1;
                    }
                    __syncthreads();
                }
            }
        }

        // what happens to each slot: 1 = complete in this tile, 2 / 3 = partial row 0 / 1 of the tile
        if (lay.leader && tlane == 0) {
            s_node[slot] = e.node;
            s_state[slot] = (first && s_last[slot] != 0) ? 1 : (lay.team == 0 ? 2 : 3);
        }
        __syncthreads();

        // ---- Update: rows of the tile times W
        for (int rt = rt_first; rt * 16 < nslots; rt += rt_step) {
            const float *arow = s_A + (size_t)(16 * rt + lrow) * LDA;
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int k = 16 * s + 4 * lk;
                const float4 a4 = *reinterpret_cast<const float4 *>(arow + k);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, wcol[(k + 0) * LDW], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, wcol[(k + 1) * LDW], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, wcol[(k + 2) * LDW], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, wcol[(k + 3) * LDW], acc, 0, 0, 0);
            }
            if (col < M) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 16 * rt + 4 * lk + i;  // result row -> slot
                    if (r < nslots) {
                        const int st = s_state[r];
                        if (st == 1) {
                            fp.out[(size_t)s_node[r] * M + col] = act_bias(acc[i], bcol, fp.relu);
                        } else if (st >= 2) {
                            __hip_atomic_store(p.part_rows + ((size_t)tile * 2 + (st - 2)) * M + col, acc[i],
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
        }

        // ---- ordered flush of the (at most two) unfinished nodes: slot 0 and the last slot
        const bool part0 = s_state[0] == 2, part1 = s_state[nslots - 1] == 3;
        if (part0 || part1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the partial rows have left this wave
            __syncthreads();                                   // ... and every other wave of the block
            if (wave == 0) {
                for (int which = 0; which < 2; ++which) {
                    if (which == 0 ? !part0 : !part1) continue;
                    const int node = s_node[which == 0 ? 0 : nslots - 1];
                    int arrived = 0;
                    if (lane == 0) arrived = atomicAdd(&p.cnt[node], 1);
                    arrived = __shfl(arrived, 0);
                    const int gfirst = p.ngptr[node], gend = p.ngptr[node + 1];
                    const int64_t b0 = gfirst / T, b1 = (gend - 1) / T;
                    if (arrived != (int)(b1 - b0)) continue;
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                    if (lane == 0) p.cnt[node] = 0;
                    if (lane < M) {
                        // in its first tile the node is the tile's first node only if it starts the tile
                        float sum = __hip_atomic_load(
                            p.part_rows + ((size_t)b0 * 2 + (gfirst % T == 0 ? 0 : 1)) * M + lane, __ATOMIC_RELAXED,
                            __HIP_MEMORY_SCOPE_AGENT);
                        for (int64_t b = b0 + 1; b <= b1; b += 4) {
                            float t[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                t[q] = 0.0f;
                                if (b + q <= b1)
                                    t[q] = __hip_atomic_load(p.part_rows + ((size_t)(b + q) * 2) * M + lane,
                                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (b + q <= b1) sum += t[q];
                        }
                        const float bl = fp.b ? fp.b[lane] : 0.0f;
                        fp.out[(size_t)node * M + lane] = act_bias(sum, bl, fp.relu);
                    }
                }
            }
        }
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

// Tries the fused GIN layer.  Returns GNN_OK after enqueueing it, 1 if the shape is outside what it
// covers (the caller then runs aggregation and GEMM separately), < 0 on error.  p.part_rows must
// point to room for 2 * tiles rows of max(K, M) floats.
int try_gin_layer_fused(AggParams &p, int vec, int wpb, const float *W, const float *b, float *out, int M, int relu,
                         int64_t tiles_upper, hipStream_t s)
{
    const int K = p.dim;
    const int ns = K <= 16 ? 1 : (K <= 32 ? 2 : (K <= 64 ? 4 : (K <= 128 ? 8 : 0)));
    const int T = p.T;
    if (vec != 4 || ns == 0 || M > 64 || T > 64 || !p.part_rows) return 1;
    const int ct = (M + 15) / 16;
    if (wpb > 8 || wpb % ct != 0) return 1;
    if (p.iter_total > 4) return 1;
    if (((uintptr_t)W | (uintptr_t)out) % 4 != 0) return 1;
    const int kp = 16 * ns, lda = kp + 4, ldw = 16 * ct + 4;
    const int a_rows = (T + 15) / 16 * 16;  // whole 16-row MFMA tiles
    size_t lds = (size_t)(kMaxWavesPerBlock + 3 * T + (size_t)T * p.ngs) * 4;
    lds = (lds + 15) & ~(size_t)15;
    lds += ((size_t)kp * ldw + (size_t)a_rows * lda + (size_t)wpb * 64) * 4;
    if (lds > kMaxLdsBytes) return 1;

    const int64_t grid = tiles_upper;
    const int64_t nchunks = ((int64_t)p.n + 63) / 64;
    int64_t extra = (nchunks + (int64_t)wpb * 8 - 1) / ((int64_t)wpb * 8);
    if (extra > 4096) extra = 4096;
    if (grid + extra >= ((int64_t)1 << 31)) return GNN_ELIMIT;

    FusedParams fp;
    fp.a = p;
    fp.a.tile_blocks = grid;
    fp.a.extra_blocks = (int)extra;
    fp.W = W;
    fp.b = b;
    fp.out = out;
    fp.M = M;
    fp.relu = relu;
    fp.ct = ct;
    fp.a_rows = a_rows;
    const void *fn = fused_fn(p.iter_total, ns);
    void *args[] = {(void *)&fp};
    GNN_HIP_TRY(hipLaunchKernel(fn, dim3((unsigned)(grid + extra)), dim3((unsigned)(wpb * 64)), args, lds, s));
    return GNN_OK;
}

}  // namespace gnn
