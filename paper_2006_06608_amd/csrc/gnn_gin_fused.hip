// GIN layer with the Update fused into the Aggregation: out = act(((1+eps) X + sum_N X) W + b) in one
// launch (an MI355X addition; the paper runs the two phases as separate kernels).  Two forms: the
// wave-tile form (k_gin_layer_fused_w, further down; rows of 16, 32 or 64 floats), in which every wave
// works on its own, and the older block-tile form for the other shapes:
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


// ---------------------------------------------------------------------------------------------------
// Wave-tile form of the fused layer, for rows that a team covers in one pass (K = ITER * dw * 4 = 16, 32
// or 64 floats) and groups of at most J * dw entries.
//
// A wave serves 16 consecutive neighbor groups on its own, in R = 16 / (teams per wave) rounds: it keeps the
// groups' column indices in registers (lane l of a team holds entries l, l + dw, ...; a shuffle hands them
// round), gathers, reduces over the teams that share a target node and leaves every target node of its 16
// groups as one row of its private 16-row LDS tile -- Algorithm 1's slots at the scale of a wave: a row
// per distinct node, a node that continues from one round into the next adding to the row it has.  The
// only thing the waves of a block share is the copy of W in LDS, which each of them helps to write
// before it gathers and which one barrier after the gather publishes.  The tile then goes through
// v_mfma_f32_16x16x4_f32 with the roles of the operands exchanged (W^T times tile^T), so that a lane ends
// up with four consecutive output columns of one node and stores 16 bytes.  Rows whose node has all its
// groups in the wave get bias and activation and go to `out`; the (at most two) others are partial sums
// and take the ordered flush in units of wave tiles: transformed partial row (M floats; the product is
// linear) to scratch, arrival counter, the wave that arrives last adds the partial rows in tile order.
// No wave waits for another one except at the one barrier.
template <int DL, int ITER, int U, int J, int NW, bool WEIGHTED, bool SELF>
__global__ __launch_bounds__(NW * 64) void k_gin_layer_fused_w(FusedParams fp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const AggParams &p = fp.a;
    const HeaderVals hv = load_header(p.hdr);
    if (!header_vals_ok(hv, p)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) note_stale(p.hdr, p);
        return;
    }
    constexpr int VEC = 4;
    constexpr int dwl = 1 << DL, G = 64 >> DL;  // lanes per team, teams per round
    constexpr int TILE = kFusedWaveTile;        // groups per wave
    constexpr int R = TILE / G;                 // rounds
    constexpr int K = ITER * dwl * VEC;
    constexpr int NS = K / 16;
    constexpr int LDA = K + 4, LDW = 68;
    static_assert(G <= TILE && K % 16 == 0 && U <= dwl * J, "shape not covered");
    const int M = fp.M, ct = fp.ct;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tlane = lane & (dwl - 1), team = lane >> DL, tbase = lane & ~(dwl - 1);
    const int lrow = lane & 15, lk = lane >> 4;

    // LDS: sW[K][LDW] | sA[NW][16][LDA] | sNode[NW][16] | sFlag[NW][16]   (blocks that serve rows without
    // entries use the tile area for their lists)
    float *sW = reinterpret_cast<float *>(smem);
    float *sA = sW + K * LDW + (size_t)wave * TILE * LDA;
    int *sNode = reinterpret_cast<int *>(sW + K * LDW + (size_t)NW * TILE * LDA) + wave * 16;
    int *sFlag = sNode + NW * 16;  // bit 0: the row holds its node's first group, bit 1: its last group

    // this thread's part of W (zero padded to 64 columns): requested early, written to LDS further down
    constexpr int NL = (K * 16 + NW * 64 - 1) / (NW * 64);
    float4 w4[NL];
    auto load_w = [&]() {
        const bool vecw = (M % 4 == 0) && (((uintptr_t)fp.W & 15) == 0);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + NW * 64 * i, k = idx >> 4, c = (idx & 15) * 4;
            w4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < K && c < M) {
                const float *src = fp.W + (size_t)k * M + c;
                if (vecw) {
                    w4[i] = *reinterpret_cast<const float4 *>(src);
                } else {
                    w4[i].x = src[0];
                    if (c + 1 < M) w4[i].y = src[1];
                    if (c + 2 < M) w4[i].z = src[2];
                    if (c + 3 < M) w4[i].w = src[3];
                }
            }
        }
    };
    auto store_w = [&]() {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + NW * 64 * i, k = idx >> 4, c = (idx & 15) * 4;
            if (k < K) *reinterpret_cast<float4 *>(sW + k * LDW + c) = w4[i];
        }
    };

    if ((int)blockIdx.x < p.extra_blocks) {
        // ---- the first blocks of the grid (a multiple of the number of XCDs): rows without entries,
        // act((1+eps) x W + b); every wave works alone, 16 such rows at a time
        int *mylist = reinterpret_cast<int *>(sA);  // 64 ints of the wave's own tile area
        const int64_t nchunks = ((int64_t)p.n + 63) / 64;
        const int64_t first_chunk = (int64_t)blockIdx.x * NW + wave;
        const int64_t chunk_stride = (int64_t)p.extra_blocks * NW;
        // a block whose nodes all have entries (every block, on many graphs) leaves without touching W
        int any = 0;
        for (int64_t c = first_chunk; c < nchunks; c += chunk_stride) {
            const int64_t v = c * 64 + lane;
            any |= (v < p.n && p.ngptr[v] == p.ngptr[v + 1]) ? 1 : 0;
        }
        if (!__syncthreads_or(any)) return;
        if (!SELF) {
            // no own-row term (GCN): a row without entries is act(b)
            for (int64_t c = first_chunk; c < nchunks; c += chunk_stride) {
                const int64_t v = c * 64 + lane;
                if (v < p.n && p.ngptr[v] == p.ngptr[v + 1])
                    for (int cc = 0; cc < M; ++cc) fp.out[(size_t)v * M + cc] = act_bias(0.0f, fp.b ? fp.b[cc] : 0.0f, fp.relu);
            }
            return;
        }
        load_w();
        store_w();
        __syncthreads();
        for (int64_t c = first_chunk; c < nchunks; c += chunk_stride) {
            const int64_t v = c * 64 + lane;
            const bool empty = v < p.n && p.ngptr[v] == p.ngptr[v + 1];
            const unsigned long long m = __ballot(empty);
            if (m == 0ull) continue;
            const int cnt = __popcll(m);
            if (empty) mylist[__popcll(m & ((1ull << lane) - 1ull))] = lane;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            for (int base = 0; base < cnt; base += 16) {
                // lane (lrow, lk) feeds node `lrow` of this group of 16, k = 16 s + 4 lk .. + 3
                const bool rok = base + lrow < cnt;
                const int64_t node = c * 64 + (rok ? mylist[base + lrow] : 0);
                float4 a4[NS];
#pragma unroll
                for (int s2 = 0; s2 < NS; ++s2) {
                    a4[s2] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (rok) a4[s2] = *reinterpret_cast<const float4 *>(p.X + (size_t)node * K + 16 * s2 + 4 * lk);
                }
                for (int t = 0; t < ct; ++t) {
                    const float *wc = sW + 16 * t + lrow;
                    f32x4 d = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s2 = 0; s2 < NS; ++s2) {
                        const int k = 16 * s2 + 4 * lk;
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 0) * LDW], a4[s2].x, d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 1) * LDW], a4[s2].y, d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 2) * LDW], a4[s2].z, d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 3) * LDW], a4[s2].w, d, 0, 0, 0);
                    }
                    // d[i] = (x W)[node lrow][16 t + 4 lk + i]
                    if (rok) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int cc = 16 * t + 4 * lk + i;
                            if (cc < M) fp.out[(size_t)node * M + cc] = act_bias(p.self_scale * d[i], fp.b ? fp.b[cc] : 0.0f, fp.relu);
                        }
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }

    load_w();
    const int64_t bid = (int64_t)blockIdx.x - p.extra_blocks;
    int64_t btile = bid;
    if (p.xcd_remap) {
        const int64_t x = bid % kNumXcd, q = bid / kNumXcd;
        btile = ((q / kXcdRun) * kNumXcd + x) * kXcdRun + q % kXcdRun;
    }
    const int64_t num_ng = hv.num_ng;
    if (btile * (NW * TILE) >= num_ng) return;  // (the whole block: the grid is sized from an upper bound)
    const int64_t wtile = btile * NW + wave;  // the wave's tile: groups [16 wtile, 16 wtile + 16)
    const int64_t g0 = wtile * TILE;

    // tuples, then own rows and column indices of all rounds: two round trips in front of the gather
    NgEntry e[R];
    bool valid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t g = g0 + r * G + team;
        valid[r] = g < num_ng;
        e[r].node = -1;
        e[r].start = e[r].end = e[r].flags = 0;
        if (valid[r]) e[r] = p.ng[g];
    }
    const float *xb = p.X + (size_t)tlane * VEC;
    int cidx[R][J];
    float cw[R][WEIGHTED ? J : 1];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int len = e[r].end - e[r].start;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int k = tlane + j * dwl;
            cidx[r][j] = k < len ? load_stream(&p.colidx[e[r].start + k]) : -1;
            if (WEIGHTED) cw[r][j] = k < len ? load_stream(&p.ew[e[r].start + k]) : 0.0f;
        }
    }
    store_w();

    int nrows = 0;           // rows of the tile in use (wave-uniform)
    int prev_last_node = -2; // target node of the last group of the round before
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int len = e[r].end - e[r].start;
        const bool first = (e[r].flags & 1) != 0;
        float acc[ITER][VEC], xs[ITER][VEC];
        // the node's own row is a term of its first group; its load does not wait for the indices and is
        // used only after the neighbour rows, so nothing waits for it alone
#pragma unroll
        for (int c = 0; c < ITER; ++c) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[c][j] = xs[c][j] = 0.0f;
            if (SELF && valid[r] && first)
                load_vec<VEC>(xs[c], xb + (size_t)(unsigned)e[r].node * (unsigned)K + c * dwl * VEC);
        }
#pragma unroll
        for (int jb = 0; jb < J * dwl / U; ++jb) {
            if (jb * U < len) {
                int col[U];
                float wgt[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = jb * U + u;  // compile-time: register k / dw, lane k % dw of the team
                    col[u] = __shfl(cidx[r][k >> DL], tbase + (k & (dwl - 1)));
                    if (WEIGHTED) wgt[u] = __shfl(cw[r][k >> DL], tbase + (k & (dwl - 1)));
                }
                float v[U][ITER][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        if (col[u] >= 0) {
                            load_vec<VEC>(v[u][c], xb + (size_t)(unsigned)col[u] * (unsigned)K + c * dwl * VEC);
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
                        for (int j = 0; j < VEC; ++j) {
                            if (WEIGHTED) acc[c][j] = fmaf(wgt[u], v[u][c][j], acc[c][j]);
                            else acc[c][j] += v[u][c][j];
                        }
            }
        }
        if (SELF) {
#pragma unroll
            for (int c = 0; c < ITER; ++c)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[c][j] = fmaf(p.self_scale, xs[c][j], acc[c][j]);
        }

        // Algorithm 1 inside the round: a team opens a segment when its target node differs from the team's
        // before it; the segment's first team collects the segment's sum and its "last group" flag
        const int prev_node = __shfl_up(e[r].node, dwl);
        const bool seg_head = valid[r] && (team == 0 || e[r].node != prev_node);
        const unsigned long long cont = __ballot(valid[r] && !seg_head);
        int flags = valid[r] ? (e[r].flags & 3) : 0;
        if (cont != 0ull) {
            const int key = valid[r] ? e[r].node : -1;
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
                const int ol = __shfl_down(flags, o);
                if (take) flags |= ol & 2;
            }
        }
        // rows: one per segment; the first segment continues the last row of the round before if it has
        // the same target node
        const unsigned long long heads = __ballot(seg_head && tlane == 0);
        const int node0 = __shfl(e[r].node, 0);
        const bool joins = r > 0 && node0 >= 0 && node0 == prev_last_node;
        // (heads before the team's own first lane: the team's own bit must not count)
        const int row = nrows + __popcll(heads & ((1ull << tbase) - 1ull)) - (joins ? 1 : 0);
        if (seg_head) {
            float *arow = sA + row * LDA;
            if (joins && team == 0) {
#pragma unroll
                for (int c = 0; c < ITER; ++c) {
                    float4 cur = *reinterpret_cast<float4 *>(arow + (c * dwl + tlane) * VEC);
                    cur.x += acc[c][0];
                    cur.y += acc[c][1];
                    cur.z += acc[c][2];
                    cur.w += acc[c][3];
                    *reinterpret_cast<float4 *>(arow + (c * dwl + tlane) * VEC) = cur;
                }
                if (tlane == 0) sFlag[row] |= flags & 2;
            } else {
#pragma unroll
                for (int c = 0; c < ITER; ++c)
                    *reinterpret_cast<float4 *>(arow + (c * dwl + tlane) * VEC) =
                        make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
                if (tlane == 0) {
                    sNode[row] = e[r].node;
                    sFlag[row] = flags;
                }
            }
        }
        nrows += __popcll(heads) - (joins ? 1 : 0);
        prev_last_node = __shfl(valid[r] ? e[r].node : -2, 63);
        // (the next round may add to a row written here: same wave, program order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    __syncthreads();  // W is complete in LDS (every wave of the block comes here)
    if (nrows == 0) return;

    // ---- Update: (tile W)^T = W^T tile^T, lane (lrow, lk) supplies tile[lrow][k] and W[k][16 t + lrow]
    float4 a4[NS];
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) {
        a4[s2] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (lrow < nrows) a4[s2] = *reinterpret_cast<const float4 *>(sA + lrow * LDA + 16 * s2 + 4 * lk);
    }
    const int rnode = lrow < nrows ? sNode[lrow] : -1;
    const int rflag = lrow < nrows ? sFlag[lrow] : 0;
    const bool complete = rflag == 3;
    // an unfinished row 0 is the tile's partial row 0, an unfinished last row its partial row 1
    float *prow = p.part_rows + ((size_t)wtile * 2 + (lrow == 0 ? 0 : 1)) * M;
    const bool vec_out = (M % 4 == 0) && (((uintptr_t)fp.out & 15) == 0);
    for (int t = 0; t < ct; ++t) {
        const float *wc = sW + 16 * t + lrow;
        f32x4 d = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) {
            const int k = 16 * s2 + 4 * lk;
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 0) * LDW], a4[s2].x, d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 1) * LDW], a4[s2].y, d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 2) * LDW], a4[s2].z, d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[(k + 3) * LDW], a4[s2].w, d, 0, 0, 0);
        }
        // d[i] = (row lrow of the tile times W)[16 t + 4 lk + i]
        const int c0 = 16 * t + 4 * lk;
        if (rnode >= 0 && c0 < M) {
            if (complete) {
                float *o = fp.out + (size_t)rnode * M + c0;
                if (vec_out) {
                    float4 r4;
                    r4.x = act_bias(d[0], fp.b ? fp.b[c0 + 0] : 0.0f, fp.relu);
                    r4.y = act_bias(d[1], fp.b ? fp.b[c0 + 1] : 0.0f, fp.relu);
                    r4.z = act_bias(d[2], fp.b ? fp.b[c0 + 2] : 0.0f, fp.relu);
                    r4.w = act_bias(d[3], fp.b ? fp.b[c0 + 3] : 0.0f, fp.relu);
                    *reinterpret_cast<float4 *>(o) = r4;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (c0 + i < M) o[i] = act_bias(d[i], fp.b ? fp.b[c0 + i] : 0.0f, fp.relu);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (c0 + i < M) __hip_atomic_store(prow + c0 + i, d[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // ---- ordered flush of the (at most two) unfinished rows: row 0 and the last row
    const int flag0 = sFlag[0], flagl = sFlag[nrows - 1];
    const bool part0 = flag0 != 3, part1 = nrows > 1 && flagl != 3;
    if (part0 || part1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the partial rows have left this wave
        for (int which = 0; which < 2; ++which) {
            if (which == 0 ? !part0 : !part1) continue;
            const int node = sNode[which == 0 ? 0 : nrows - 1];
            int arrived = 0;
            if (lane == 0) arrived = atomicAdd(&p.cnt[node], 1);
            arrived = __shfl(arrived, 0);
            const int gfirst = p.ngptr[node], gend = p.ngptr[node + 1];
            const int64_t b0 = gfirst / TILE, b1 = (gend - 1) / TILE;
            if (arrived != (int)(b1 - b0)) continue;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            if (lane == 0) p.cnt[node] = 0;
            if (lane < M) {
                // in its first tile the node is the tile's first node only if it starts the tile
                float sum = __hip_atomic_load(p.part_rows + ((size_t)b0 * 2 + (gfirst % TILE == 0 ? 0 : 1)) * M + lane,
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int64_t b = b0 + 1; b <= b1; b += 4) {
                    float tq[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        tq[q] = 0.0f;
                        if (b + q <= b1)
                            tq[q] = __hip_atomic_load(p.part_rows + ((size_t)(b + q) * 2) * M + lane, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (b + q <= b1) sum += tq[q];
                }
                fp.out[(size_t)node * M + lane] = act_bias(sum, fp.b ? fp.b[lane] : 0.0f, fp.relu);
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

// ---- the wave-tile form ----
// Waves per block (they share the copy of W): 8 on large graphs, where the copy is what limits the number of
// resident waves; 4 when the whole grid is resident at once anyway, so that more blocks spread over the CUs.
constexpr int kFusedWavesLarge = 8, kFusedWavesSmall = 4;
constexpr int64_t kFusedSmallGrid = 4096;  // wave tiles

template <int DL, int ITER, int U, int NW, bool WEIGHTED, bool SELF>
static const void *fused_w_fn(int j)
{
    if (j <= 2) return (const void *)k_gin_layer_fused_w<DL, ITER, U, 2, NW, WEIGHTED, SELF>;
    if (j <= 4) return (const void *)k_gin_layer_fused_w<DL, ITER, U, 4, NW, WEIGHTED, SELF>;
    if constexpr (DL == 2 && ITER == 1) {  // rows of 16 floats: groups of up to 32 entries
        if (j <= 8) return (const void *)k_gin_layer_fused_w<DL, ITER, U, 8, NW, WEIGHTED, SELF>;
    }
    return nullptr;
}

// Kernel for (team width 2^dl, chunks per lane, registers of indices per lane), or null if not covered.
template <int NW, bool WEIGHTED, bool SELF>
static const void *fused_w_kernel_nw(int dl, int iter, int j)
{
    if (dl == 3 && iter == 2) return fused_w_fn<3, 2, 4, NW, WEIGHTED, SELF>(j);  // K = 64, teams of 8
    if (dl == 4 && iter == 1) return fused_w_fn<4, 1, 8, NW, WEIGHTED, SELF>(j);  // K = 64, teams of 16
    if (dl == 3 && iter == 1) return fused_w_fn<3, 1, 8, NW, WEIGHTED, SELF>(j);  // K = 32, teams of 8
    if (dl == 2 && iter == 2) return fused_w_fn<2, 2, 4, NW, WEIGHTED, SELF>(j);  // K = 32, teams of 4
    if (dl == 2 && iter == 1) return fused_w_fn<2, 1, 8, NW, WEIGHTED, SELF>(j);  // K = 16, teams of 4
    return nullptr;
}

// gcn: edge weights, no own-row term (Eq. 2); otherwise GIN: no weights, own row scaled by 1 + eps (Eq. 3)
static const void *fused_w_kernel(bool gcn, int dl, int iter, int j, int nw = kFusedWavesLarge)
{
    if (gcn)
        return nw == kFusedWavesSmall ? fused_w_kernel_nw<kFusedWavesSmall, true, false>(dl, iter, j)
                                      : fused_w_kernel_nw<kFusedWavesLarge, true, false>(dl, iter, j);
    return nw == kFusedWavesSmall ? fused_w_kernel_nw<kFusedWavesSmall, false, true>(dl, iter, j)
                                  : fused_w_kernel_nw<kFusedWavesLarge, false, true>(dl, iter, j);
}

bool gin_layer_fused_wave_tiles(const AggParams &p, int vec, int M)
{
    if (vec != 4 || !p.full_rows || M > 64 || M < 1) return false;
    const int dwl = 1 << p.dwl_log2;
    return fused_w_kernel(p.ew != nullptr, p.dwl_log2, p.iter_total, (p.ngs + dwl - 1) / dwl) != nullptr;
}

static int launch_gin_layer_fused_w(AggParams &p, const float *W, const float *b, float *out, int M, int relu,
                                    int64_t ng_cap, hipStream_t s, int *waves_used)
{
    const int dwl = 1 << p.dwl_log2;
    const int K = p.dim;
    const int64_t wave_tiles = (ng_cap + kFusedWaveTile - 1) / kFusedWaveTile;
    const int nw = wave_tiles <= kFusedSmallGrid ? kFusedWavesSmall : kFusedWavesLarge;
    const void *fn = fused_w_kernel(p.ew != nullptr, p.dwl_log2, p.iter_total, (p.ngs + dwl - 1) / dwl, nw);
    if (!fn || !p.part_rows || ((uintptr_t)W | (uintptr_t)out) % 4 != 0) return 1;
    const size_t lds = ((size_t)K * 68 + (size_t)nw * kFusedWaveTile * (K + 4) + (size_t)nw * 32) * 4;
    if (lds > kMaxLdsBytes) return 1;
    int64_t grid = (wave_tiles + nw - 1) / nw;
    if (p.xcd_remap) grid = (grid + kNumXcd * kXcdRun - 1) / (kNumXcd * kXcdRun) * (kNumXcd * kXcdRun);
    const int64_t nchunks = ((int64_t)p.n + 63) / 64;
    // rows without entries: the first blocks of the grid, each wave taking about two 64-node chunks
    int64_t extra = (nchunks + (int64_t)nw * 2 - 1) / ((int64_t)nw * 2);
    if (extra > 8192) extra = 8192;
    extra = (extra + kNumXcd - 1) / kNumXcd * kNumXcd;
    if (grid + extra >= ((int64_t)1 << 31)) return GNN_ELIMIT;
    FusedParams fp;
    fp.a = p;
    fp.a.T = kFusedWaveTile;
    fp.a.tile_blocks = grid;
    fp.a.extra_blocks = (int)extra;
    fp.W = W;
    fp.b = b;
    fp.out = out;
    fp.M = M;
    fp.relu = relu;
    fp.ct = (M + 15) / 16;
    fp.a_rows = 16;
    void *args[] = {(void *)&fp};
    GNN_HIP_TRY(hipLaunchKernel(fn, dim3((unsigned)(grid + extra)), dim3((unsigned)(nw * 64)), args, lds, s));
    if (waves_used) *waves_used = nw;
    return GNN_OK;
}

// Tries the fused GIN layer.  Returns GNN_OK after enqueueing it, 1 if the shape is outside what it
// covers (the caller then runs aggregation and GEMM separately), < 0 on error.  p.part_rows must
// point to room for 2 * tiles rows of max(K, M) floats.
int try_gin_layer_fused(AggParams &p, int vec, int wpb, const float *W, const float *b, float *out, int M, int relu,
                         int64_t tiles_upper, hipStream_t s, int *waves_used)
{
    if (waves_used) *waves_used = wpb;
    if (p.T == kFusedWaveTile && gin_layer_fused_wave_tiles(p, vec, M)) {
        // (the caller sized the partial rows for tiles of 16 groups)
        return launch_gin_layer_fused_w(p, W, b, out, M, relu, tiles_upper * kFusedWaveTile, s, waves_used);
    }
    if (p.ew) return 1;  // (the block-tile form has no edge weights)
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
