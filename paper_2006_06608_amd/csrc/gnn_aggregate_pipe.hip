// Persistent, software-pipelined form of the aggregation kernel (Sec. 4 + Sec. 5.2) for gfx950.
//
// Same mapping as k_aggregate (team of dwl lanes per neighbor group, 64/dwl teams per wavefront,
// T = W*64/dwl groups per block, LDS slots per Algorithm 1, leader flush), with the launch
// shaped for latency: a fixed number of resident blocks walk over the tiles, and while the
// neighbor rows of tile i are in flight the tuples of tile i+2 and the column indices / edge
// weights of tile i+1 are already being fetched.  In steady state a tile costs one global
// round trip (the row reads) and one block barrier (before the leader flush); the LDS slot and
// index buffers are double-buffered so that no second barrier is needed.
//
// Requirements checked by the host: T <= 64 (one tuple per lane describes the whole tile, so
// every wave derives Algorithm 1's slots and leaders with ballots, without talking to the other
// waves) and 64/dwl * ngs <= 64 * kPipeIdxLoads (a wave's index range fits the prefetch registers).
#include <hip/hip_runtime.h>

#include "gnn_launch.h"
#include "gnn_pipe_common.h"

namespace gnn {

constexpr int kPipeMinTilesPerBlock = 4;  // below this the pipeline never reaches steady state

template <int VEC, int ITER, int U, bool WEIGHTED, bool SELF>
__global__ __launch_bounds__(1024) void k_aggregate_pipe(AggParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const WsHeader *hdr = p.hdr;
    if (!header_ok(hdr, p)) return;

    const int T = p.T, dim = p.dim, ngs = p.ngs;
    const int64_t num_ng = hdr->num_ng;
    const int64_t tiles = (num_ng + T - 1) / T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int dwl_log2 = p.dwl_log2, dwl = 1 << dwl_log2;
    const int G = 64 >> dwl_log2;
    const int tlane = lane & (dwl - 1);
    const int team_in_wave = lane >> dwl_log2;
    const int wcap = G * ngs;  // index entries of one wave

    // LDS: [2][T*dim] slots | [2][T] "saw the node's last group" | [2][nwaves][wcap] indices | same, weights
    float *s_slot = reinterpret_cast<float *>(smem);
    int *s_last = reinterpret_cast<int *>(s_slot + 2 * (size_t)T * dim);
    int *s_col = s_last + 2 * T;
    float *s_w = reinterpret_cast<float *>(s_col + 2 * (size_t)nwaves * wcap);
    int *s_list = reinterpret_cast<int *>(s_w + (WEIGHTED ? 2 * (size_t)nwaves * wcap : 0));  // [nwaves][64]

    for (int i = tid; i < 2 * T * dim; i += blockDim.x) s_slot[i] = 0.0f;
    for (int i = tid; i < 2 * T; i += blockDim.x) s_last[i] = 0;
    __syncthreads();

    // tile schedule: with the XCD-aware order, the blocks of one XCD (blockIdx % 8) take a run of
    // consecutive tiles in every round, so neighbouring target nodes share that XCD's L2
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
    float wpre[kPipeIdxLoads];
    auto prefetch_idx = [&](const TileView &V) {
#pragma unroll
        for (int r = 0; r < kPipeIdxLoads; ++r) {
            const int k = lane + 64 * r;
            cpre[r] = 0;
            wpre[r] = 0.0f;
            if (k < V.ws1 - V.ws0) {
                cpre[r] = load_stream(&p.colidx[V.ws0 + k]);
                if (WEIGHTED) wpre[r] = load_stream(&p.ew[V.ws0 + k]);
            }
        }
    };
    auto commit_idx = [&](const TileView &V, int buf) {
        int *dc = s_col + ((size_t)buf * nwaves + wave) * wcap;
        float *dw = s_w + ((size_t)buf * nwaves + wave) * wcap;
#pragma unroll
        for (int r = 0; r < kPipeIdxLoads; ++r) {
            const int k = lane + 64 * r;
            if (k < V.ws1 - V.ws0) {
                dc[k] = cpre[r];
                if (WEIGHTED) dw[k] = wpre[r];
            }
        }
    };

    // prologue: tile 0 staged synchronously, tuples of tile 1 in flight
    NgEntry tl_next = fetch_tuples(tile_of(1));
    TileView cur = derive_tile(fetch_tuples(tile_of(0)), dwl_log2, T);
    prefetch_idx(cur);
    commit_idx(cur, 0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    for (int64_t it = 0;; ++it) {
        if (tile_of(it) >= tiles) break;  // same for every wave of the block
        const int buf = (int)(it & 1);
        // fetch ahead: tuples of tile it+2, indices of tile it+1
        const NgEntry tl_after = fetch_tuples(tile_of(it + 2));
        const TileView nxt = derive_tile(tl_next, dwl_log2, T);
        prefetch_idx(nxt);

        const NgEntry e = cur.e;
        const int len = cur.valid ? e.end - e.start : 0;
        const int off = e.start - cur.ws0;
        const bool first = (e.flags & 1) != 0;
        const int *lc = s_col + ((size_t)buf * nwaves + wave) * wcap + off;
        const float *lw = s_w + ((size_t)buf * nwaves + wave) * wcap + off;
        float *slots = s_slot + (size_t)buf * T * dim;
        int *lastf = s_last + buf * T;

        const unsigned long long cont = __ballot(cur.valid && !cur.leader && team_in_wave > 0);
        const bool seg_head = cur.valid && (team_in_wave == 0 || cur.leader);
        int lastflag = cur.valid ? (e.flags & 2) : 0;
        bool lastflag_done = false;
        bool complete_in_wave = false;

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
                int col[U];
                float w[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = base + u;
                    const bool a = k < len;
                    col[u] = a ? lc[k] : -1;
                    if (WEIGHTED) w[u] = a ? lw[k] : 0.0f;
                }
                float v[U][ITER][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        if (col[u] >= 0 && dok[c]) {
                            load_vec<VEC>(v[u][c], xb + (size_t)col[u] * dim + (size_t)c * dwl * VEC);
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
                            if (WEIGHTED) acc[c][j] = fmaf(w[u], v[u][c][j], acc[c][j]);
                            else acc[c][j] += v[u][c][j];
                        }
            }

            // segmented reduction over the teams of this wave that share a target node
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
            complete_in_wave = seg_head && first && lastflag != 0;

            if (seg_head) {
                if (complete_in_wave) {
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        const int d = ((c0 + c) * dwl + tlane) * VEC;
                        if (d < dim) {
                            float r[VEC];
                            if (SELF) {
                                float xs[VEC];
                                load_vec<VEC>(xs, p.X + (size_t)e.node * dim + d);
#pragma unroll
                                for (int j = 0; j < VEC; ++j) r[j] = fmaf(p.self_scale, xs[j], acc[c][j]);
                            } else {
#pragma unroll
                                for (int j = 0; j < VEC; ++j) r[j] = acc[c][j];
                            }
#pragma unroll
                            for (int j = 0; j < VEC; ++j) r[j] = epilogue(r[j], p.bias, d + j, p.relu);
                            if (p.stream_out) store_vec_stream<VEC>(p.out + (size_t)e.node * dim + d, r);
                            else store_vec<VEC>(p.out + (size_t)e.node * dim + d, r);
                        }
                    }
                } else {
                    float *srow = slots + (size_t)cur.slot * dim;
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        const int d = ((c0 + c) * dwl + tlane) * VEC;
                        if (d < dim) {
#pragma unroll
                            for (int j = 0; j < VEC; ++j) atomicAdd(&srow[d + j], acc[c][j]);
                        }
                    }
                    if (lastflag != 0 && tlane == 0) lastf[cur.slot] = 1;
                }
            }
        }
        __syncthreads();

        // leader flush (Algorithm 1); the leader also clears its slot for the tile after next
        if (cur.leader && !complete_in_wave) {
            const bool complete = first && lastf[cur.slot] != 0;
            float *srow = slots + (size_t)cur.slot * dim;
            float *orow = p.out + (size_t)e.node * dim;
            for (int c = 0; c < p.iter_total; ++c) {
                const int d = (c * dwl + tlane) * VEC;
                if (d >= dim) break;
                float r[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    r[j] = srow[d + j];
                    srow[d + j] = 0.0f;
                }
                if (SELF && first) {
                    float xs[VEC];
                    load_vec<VEC>(xs, p.X + (size_t)e.node * dim + d);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) r[j] = fmaf(p.self_scale, xs[j], r[j]);
                }
                if (complete) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) r[j] = epilogue(r[j], p.bias, d + j, p.relu);
                    if (p.stream_out) store_vec_stream<VEC>(orow + d, r);
                    else store_vec<VEC>(orow + d, r);
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) atomicAdd(&orow[d + j], r[j]);
                }
            }
            if (tlane == 0) lastf[cur.slot] = 0;
        }

        // indices of the next tile go to the other buffer (private to this wave)
        commit_idx(nxt, buf ^ 1);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        cur = nxt;
        tl_next = tl_after;
    }

    // rows without any entry
    if (p.do_empty) write_empty_rows<VEC, SELF>(p, b * nwaves + wave, B * nwaves, s_list + wave * 64);
}

template <int VEC, int ITER, int U>
static const void *pipe_fn3(bool weighted, bool self)
{
    if (self) return (const void *)k_aggregate_pipe<VEC, ITER, U, false, true>;
    if (weighted) return (const void *)k_aggregate_pipe<VEC, ITER, U, true, false>;
    return (const void *)k_aggregate_pipe<VEC, ITER, U, false, false>;
}

template <int VEC>
static const void *pipe_fn2(int iter, bool weighted, bool self)
{
    // U neighbor rows in flight per lane, sized so that U*ITER*VEC stays near 32 registers
    constexpr int U1 = 8, U2 = VEC == 4 ? 4 : 8, U3 = 4, U4 = VEC == 4 ? 2 : 4;
    switch (iter) {
        case 1: return pipe_fn3<VEC, 1, U1>(weighted, self);
        case 2: return pipe_fn3<VEC, 2, U2>(weighted, self);
        case 3: return pipe_fn3<VEC, 3, U3>(weighted, self);
        default: return pipe_fn3<VEC, 4, U4>(weighted, self);
    }
}

static const void *pipe_fn(int vec, int iter, bool weighted, bool self)
{
    if (vec == 4) return pipe_fn2<4>(iter, weighted, self);
    if (vec == 2) return pipe_fn2<2>(iter, weighted, self);
    return pipe_fn2<1>(iter, weighted, self);
}

// LDS bytes of the pipelined kernel, or 0 if (T, ngs, dwl) do not meet its requirements.
size_t pipe_lds_bytes(int T, int dim, int ngs, int dwl_log2, int wpb, bool weighted)
{
    const int G = 64 >> dwl_log2;
    if (T > 64) return 0;
    if ((int64_t)G * ngs > 64 * kPipeIdxLoads) return 0;
    size_t b = 2 * (size_t)T * dim * 4 + 2 * (size_t)T * 4 + 2 * (size_t)wpb * G * ngs * 4 * (weighted ? 2 : 1) +
               (size_t)wpb * 64 * 4;
    return b;
}

// Number of persistent blocks to launch; 0 = too few tiles for the pipeline to pay (use the
// one-block-per-tile kernel); < 0 = error code.
int pipe_blocks(int vec, int iter, bool weighted, bool self, int cus, int wpb, size_t lds, int64_t tiles_upper, int n)
{
    int per_cu = 0;
    GNN_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pipe_fn(vec, iter, weighted, self), wpb * 64, lds));
    if (per_cu < 1) return GNN_ELIMIT;
    int64_t blocks = (int64_t)per_cu * cus;
    if (tiles_upper > 0 && tiles_upper < kPipeMinTilesPerBlock * blocks) return 0;
    if (tiles_upper <= 0) {
        // no entries at all: only the rows without entries are written
        const int64_t for_empty = ((int64_t)n + 64 * wpb - 1) / (64 * wpb);
        if (blocks > for_empty) blocks = for_empty;
    }
    if (blocks >= kNumXcd) blocks = blocks / kNumXcd * kNumXcd;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

int launch_aggregate_pipe(int vec, int iter, bool weighted, bool self, int blocks, int wpb, size_t lds, hipStream_t s,
                          AggParams &p)
{
    void *args[] = {(void *)&p};
    GNN_HIP_TRY(hipLaunchKernel(pipe_fn(vec, iter, weighted, self), dim3((unsigned)blocks), dim3((unsigned)(wpb * 64)),
                                args, lds, s));
    return GNN_OK;
}

}  // namespace gnn
