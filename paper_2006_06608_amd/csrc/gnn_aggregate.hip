// The aggregation kernels (Sec. 4 and Sec. 5.2) for gfx950, and the entry points built on them.
//
// Mapping.  A neighbor group (<= ngs consecutive CSR entries of one target node, Sec. 4.1) is
// served by a team of dwl lanes (the dimension workers of Sec. 4.2); a 64-lane wavefront carries
// 64/dwl teams side by side, so no lane idles when a row is shorter than a wavefront.  Each lane
// owns VEC consecutive floats of up to ITER chunks of the row and reads them with one 4*VEC-byte
// load per neighbor, U neighbors in flight.  A block of W waves serves T = W*64/dwl consecutive
// groups; their CSR positions are contiguous, so the block stages that index range (and the edge
// weights) in LDS with coalesced loads first.
//
// Reduction.  Teams of one wave that share a target node are combined with wavefront shuffles
// (segmented reduction).  A node whose groups all sit in one wave is then stored straight from
// registers.  Other nodes are accumulated in the block's LDS slots laid out as Algorithm 1
// prescribes; after a barrier the leader team of each slot writes the row: a plain store when
// the block saw all groups of the node.  Nodes whose groups span several blocks (high-degree ones)
// are finished in one of two ways:
//   * ordered flush (default when the workspace has room for partial rows): no float atomics.  The
//     waves of a block add to a slot in wave order; the leader stores the block's partial row to
//     scratch memory with device-coherent stores and counts itself in on the node's arrival counter;
//     the block that arrives last adds the partial rows in block order, applies bias/activation and
//     writes the row.  One launch, bitwise reproducible.
//   * atomic flush (Sec. 5.2 as printed; GNN_FLAG_ATOMIC_FLUSH or no room): the leader adds its
//     partial row to global memory with one float atomic per element; those rows are zeroed by a
//     small kernel that runs first and get bias/activation from one that runs last.
// Rows without any entry are written by blocks appended to the grid of the main kernel.  GIN's
// own-row term enters the sum with the first group of each node.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "gnn_bench.h"
#include "gnn_launch.h"

namespace gnn {

// Rows the main kernel will not store plainly: rows without entries get their final value, rows
// whose groups span several blocks are zeroed for the atomic adds.  One wave scans 64 nodes.
template <bool SELF>
__global__ __launch_bounds__(256) void k_agg_init(AggParams p)
{
    WsHeader *hdr = p.hdr;
    if (!header_ok(hdr, p)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) note_stale(hdr, p);
        return;
    }
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t v = wave * 64 + lane;
    int action = 0;
    if (v < p.n) {
        const int c0 = p.ngptr[v], c1 = p.ngptr[v + 1];
        if (c1 == c0) action = p.do_empty ? 0 : 2;
        else if (c0 / p.T != (c1 - 1) / p.T) action = 1;
    }
    unsigned long long m = __ballot(action != 0);
    while (m) {
        const int l = __ffsll((long long)m) - 1;
        m &= m - 1;
        const int act = __shfl(action, l);
        const int64_t node = wave * 64 + l;
        float *row = p.out + (size_t)node * p.dim;
        const float *xrow = p.X + (size_t)node * p.dim;
        for (int d = lane; d < p.dim; d += 64) {
            float val = 0.0f;
            if (act == 2) {
                if (SELF) val = p.self_scale * xrow[d];
                val = epilogue(val, p.bias, d, p.relu);
            }
            row[d] = val;
        }
    }
}

// Bias/activation for the rows that were completed by atomic adds.
__global__ __launch_bounds__(256) void k_agg_epilogue_spanning(AggParams p)
{
    if (!header_ok(p.hdr, p)) return;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t v = wave * 64 + lane;
    int action = 0;
    if (v < p.n) {
        const int c0 = p.ngptr[v], c1 = p.ngptr[v + 1];
        if (c1 > c0 && c0 / p.T != (c1 - 1) / p.T) action = 1;
    }
    unsigned long long m = __ballot(action != 0);
    while (m) {
        const int l = __ffsll((long long)m) - 1;
        m &= m - 1;
        float *row = p.out + (size_t)(wave * 64 + l) * p.dim;
        for (int d = lane; d < p.dim; d += 64) row[d] = epilogue(row[d], p.bias, d, p.relu);
    }
}


// The gather of one team (Sec. 4.2: the team's lanes are the dimension workers of one neighbor group):
// for the ITER chunks that start at chunk c0, acc[c][:] = reduce over the group's staged entries of
// w * X[col, chunk c].  U neighbour rows are in flight per lane.  GIN's own row (SELF, first group of
// the node) is one more term of the first batch, so no load waits for another.
// EVEC: every stored entry carries a vector of dim floats (Sec. 3.1, aggregation with edge features); the
// neighbour row is multiplied by it elementwise.  The vectors of a group are consecutive rows of E starting
// at erow0, read once, in order.
template <int VEC, int ITER, int U, bool WEIGHTED, bool SELF, int OP, bool FULL, bool EVEC = false>
__device__ __forceinline__ void gather_rows(float (&acc)[ITER][VEC], const float *__restrict__ X, const int *lc,
                                            const float *lw, int len, int node, bool self_term, float self_scale,
                                            int dim, int dwl, int tlane, int c0, const float *__restrict__ erow0 = nullptr)
{
    bool dok[ITER];
    const float *xb = X + (size_t)(c0 * dwl + tlane) * VEC;
#pragma unroll
    for (int c = 0; c < ITER; ++c) {
        dok[c] = FULL ? true : ((c0 + c) * dwl + tlane) * VEC < dim;
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[c][j] = op_identity<OP>();
    }
    // entry -1 stands for the node's own row
    for (int base = (SELF && self_term) ? -1 : 0; base < len; base += U) {
        int col[U];
        float w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // read first, select after: positions past the group still lie inside the staged area
            const int k = base + u;
            const bool a = k < len;
            const int cu = lc[k < 0 ? 0 : k];
            col[u] = a ? cu : -1;
            if (SELF && k < 0) col[u] = node;
            if (WEIGHTED) {
                const float wu = lw[k < 0 ? 0 : k];
                w[u] = a ? wu : 0.0f;
            }
            if (SELF) w[u] = k < 0 ? self_scale : 1.0f;
        }
        float v[U][ITER][VEC];
        float ev[EVEC ? U : 1][ITER][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (col[u] >= 0) {
                // 32 x 32 -> 64-bit product: one multiply-add per address
                const float *row = xb + (size_t)(unsigned)col[u] * (unsigned)dim;
                const float *er = EVEC ? erow0 + (size_t)(unsigned)(base + u) * (unsigned)dim + (size_t)(c0 * dwl + tlane) * VEC : nullptr;
#pragma unroll
                for (int c = 0; c < ITER; ++c) {
                    if (dok[c]) {
                        load_vec<VEC>(v[u][c], row + (size_t)c * dwl * VEC);
                        if (EVEC) load_vec_stream<VEC>(ev[u][c], er + (size_t)c * dwl * VEC);
                    } else {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) {
                            v[u][c][j] = op_identity<OP>();
                            if (EVEC) ev[u][c][j] = 0.0f;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int c = 0; c < ITER; ++c)
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        v[u][c][j] = op_identity<OP>();
                        if (EVEC) ev[u][c][j] = 0.0f;
                    }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int c = 0; c < ITER; ++c)
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    if (EVEC) acc[c][j] = fmaf(ev[u][c][j], v[u][c][j], acc[c][j]);
                    else if (WEIGHTED || SELF) acc[c][j] = fmaf(w[u], v[u][c][j], acc[c][j]);
                    else acc[c][j] = op_combine<OP>(acc[c][j], v[u][c][j]);
                }
    }
}

// A finished row: bias / activation / mean scaling, then the store.
template <int VEC, int ITER>
__device__ __forceinline__ void store_row(const AggParams &p, const float (&acc)[ITER][VEC], int node, int dwl, int tlane,
                                          int c0)
{
    float *orow = p.out + (size_t)node * p.dim;
    if (p.plain_rows) {
        // no bias, no activation, no scaling, rows of whole cache lines: the common aggregation
#pragma unroll
        for (int c = 0; c < ITER; ++c) {
            const int d = ((c0 + c) * dwl + tlane) * VEC;
            if (d < p.dim) store_vec_stream<VEC>(orow + d, acc[c]);
        }
        return;
    }
    const float rs = row_scale(p, node);
#pragma unroll
    for (int c = 0; c < ITER; ++c) {
        const int d = ((c0 + c) * dwl + tlane) * VEC;
        if (d < p.dim) {
            float r[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) r[j] = epilogue(acc[c][j] * rs, p.bias, d + j, p.relu);
            if (p.stream_out) store_vec_stream<VEC>(orow + d, r);
            else store_vec<VEC>(orow + d, r);
        }
    }
}

// The kernel is wave-autonomous: a wave loads the tuples of its own teams, stages their column indices
// in its own part of the LDS, gathers, reduces over the teams that share a target node with shuffles and
// stores every node whose groups all sit in the wave straight from registers -- no block barrier on
// that path, and a wave that has nothing else to do ends there.
// Only a node whose groups straddle a wave boundary inside the block takes the block-level path of
// Sec. 5.2: every wave that such a node continues into leaves its part of the sum in its LDS slot and
// meets the node's leader (Algorithm 1: the node's first team in the block) at a barrier, after which
// the leader adds the slots in wave order and flushes.  Which waves take part follows from the tuples
// a wave holds itself: a wave whose first team does not start its node continues a node of the wave
// before; a leader whose node reaches the end of the wave without its last group is continued behind
// it.  Waves that do not take part have ended by then, and the barrier counts only the waves of the
// workgroup that still run (s_barrier waits for the surviving waves of its group).
//
// DL >= 0 fixes the team width at compile time (dw = 2^DL lanes), which turns the per-load address
// arithmetic into constants; DL = -1 takes it from the launch parameters.  FULL: the row is covered in one
// pass with every lane of a team in range (dim == ITER * dw * VEC), so no lane needs a bounds check.
// The sums over 16-byte loads of such rows get (DL, FULL = true); everything else (narrow loads, rows
// that leave lanes idle or need several passes, max / min) runs the (DL = -1, FULL = false) form.
template <int VEC, int ITER, int U, int DL, bool WEIGHTED, bool SELF, int OP, bool FULL, bool EVEC = false>
__global__ __launch_bounds__(1024) void k_aggregate(AggParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int T = p.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int dim = p.dim, ngs = p.ngs;

    const HeaderVals hv = load_header(p.hdr);
    if (!header_vals_ok(hv, p)) {
        // with the ordered flush no kernel runs before this one: record why nothing was computed
        if (p.part_rows && blockIdx.x == 0 && threadIdx.x == 0) note_stale(p.hdr, p);
        return;
    }

    // LDS carve-up: staged indices [T*ngs + kStagePad] (and as many weights) | one slot of dim floats per
    // wave | three flags per wave | list of rows without entries [nw][64]
    int *s_col = reinterpret_cast<int *>(smem);
    float *s_w = reinterpret_cast<float *>(s_col + (size_t)T * ngs + kStagePad);
    size_t off_slot = ((size_t)T * ngs + kStagePad) * (WEIGHTED ? 2 : 1) * 4;
    off_slot = (off_slot + 15) & ~(size_t)15;
    float *s_slot = reinterpret_cast<float *>(smem + off_slot);   // [nw][dim]
    int *s_last = reinterpret_cast<int *>(s_slot + (size_t)nw * dim);  // [16]: the slot's part holds the node's last group
    int *s_more = s_last + kMaxWavesPerBlock;                     // [16]: the node continues behind this wave
    int *s_list = s_more + kMaxWavesPerBlock;                     // [nw][64]

    if ((int)blockIdx.x < p.extra_blocks) {
        // the first blocks of the grid: rows without entries (independent of every tile; first, so that their
        // dependent steps do not run as a tail after the last tile; a multiple of the number of XCDs, so that
        // block b - extra_blocks still runs on XCD b mod 8)
        write_empty_rows<VEC, SELF>(p, (int64_t)blockIdx.x * nw + wave, (int64_t)p.extra_blocks * nw, s_list + wave * 64);
        return;
    }
    const int64_t bid = (int64_t)blockIdx.x - p.extra_blocks;
    int64_t tile = bid;
    if (p.xcd_remap) {
        // Blocks are dealt to the eight XCDs round-robin by index.  Give every XCD runs of kXcdRun
        // consecutive tiles (neighbouring node ids, hence shared neighbours after renumbering, meet
        // in one L2) while the runs themselves still interleave over the XCDs, which keeps the
        // load balanced.
        const int64_t x = bid % kNumXcd, q = bid / kNumXcd;
        tile = ((q / kXcdRun) * kNumXcd + x) * kXcdRun + q % kXcdRun;
    }
    const int64_t num_ng = hv.num_ng;
    const int64_t g0 = tile * T;
    if (g0 >= num_ng) return;  // (the grid is sized from an upper bound of the group count)

    const int dwl_log2 = DL >= 0 ? DL : p.dwl_log2;
    const int dwl = 1 << dwl_log2, G = 64 >> dwl_log2;
    const int tlane = lane & (dwl - 1);
    const int team_in_wave = lane >> dwl_log2;
    const int team = wave * G + team_in_wave;
    const int64_t g = g0 + team;
    const bool valid = g < num_ng;

    NgEntry e;
    e.node = -1;
    e.start = e.end = e.flags = 0;
    if (valid) e = p.ng[g];
    const int len = e.end - e.start;
    const bool first = (e.flags & 1) != 0;

    // Stage the wave's indices: its teams' groups are consecutive, so their entries form one CSR range
    // [ws0, ws1), which the 64 lanes copy with coalesced loads, four requests in flight per lane.
    const int nvalid = __popcll(__ballot(valid)) >> dwl_log2;  // valid teams are a prefix of the wave
    const int ws0 = __shfl(e.start, 0);
    const int ws1 = __shfl(e.end, nvalid > 0 ? (nvalid << dwl_log2) - 1 : 0);
    const int wn = nvalid > 0 ? ws1 - ws0 : 0;
    int *wc = s_col + (size_t)wave * G * ngs;
    float *ww = s_w + (size_t)wave * G * ngs;
    for (int i0 = lane; i0 < wn; i0 += 256) {
        int ci[4];
        float wi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = i0 + 64 * q;
            ci[q] = 0;
            wi[q] = 0.0f;
            if (i < wn) {
                ci[q] = load_stream(&p.colidx[ws0 + i]);
                if (WEIGHTED) wi[q] = load_stream(&p.ew[ws0 + i]);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = i0 + 64 * q;
            if (i < wn) {
                wc[i] = ci[q];
                if (WEIGHTED) ww[i] = wi[q];
            }
        }
    }
    const int *lc = wc + (valid ? e.start - ws0 : 0);
    const float *lw = ww + (valid ? e.start - ws0 : 0);
    // (the wave reads back only what it wrote itself: program order suffices, no block barrier)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    int lastflag = valid ? (e.flags & 2) : 0;
    bool lastflag_done = false;
    bool spans_blocks = false;  // leader of a node that other tiles hold parts of
    int block_last = 0;         // leader: a wave behind this one holds the node's last group

    for (int c0 = 0; c0 < (FULL ? 1 : p.iter_total); c0 += ITER) {
        float acc[ITER][VEC];
        gather_rows<VEC, ITER, U, WEIGHTED, SELF, OP, FULL, EVEC>(acc, p.X, lc, lw, len, e.node, first && len > 0, p.self_scale,
                                                                  dim, dwl, tlane, c0,
                                                                  EVEC ? p.evec + (size_t)(unsigned)e.start * (unsigned)dim : nullptr);

        // Algorithm 1 inside the wave: a team opens a segment when its target node differs from the team's
        // before it; the segment's first team collects the segment's sum
        const int prev_node = __shfl_up(e.node, dwl);
        const bool seg_head = valid && (team_in_wave == 0 || e.node != prev_node);
        const unsigned long long cont = __ballot(valid && !seg_head);
        const int wave_last_node = __shfl(valid ? e.node : -2, 63);  // target node of the wave's last team
        // the wave's first team continues a node of the wave before it (inside the block)
        const bool from_prev = seg_head && team_in_wave == 0 && wave > 0 && !first;
        const bool leader = seg_head && !from_prev;  // Algorithm 1: first team of its (block, node) pair

        // segmented reduction over the teams of this wave that share a target node
        if (cont != 0ull) {
            const int key = valid ? e.node : -1;
            for (int o = dwl; o < 64; o <<= 1) {
                const int okey = __shfl_down(key, o);
                const bool take = (lane + o < 64) && key >= 0 && okey == key;
#pragma unroll
                for (int c = 0; c < ITER; ++c)
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        const float ov = __shfl_down(acc[c][j], o);
                        if (take) acc[c][j] = op_combine<OP>(acc[c][j], ov);
                    }
                if (!lastflag_done) {
                    const int ol = __shfl_down(lastflag, o);
                    if (take) lastflag |= ol;
                }
            }
        }
        lastflag_done = true;
        const bool complete_in_wave = seg_head && first && lastflag != 0;
        float *orow = p.out + (size_t)(valid ? e.node : 0) * dim;

        // all groups of the node sat in this wave: store from registers
        if (complete_in_wave) store_row<VEC, ITER>(p, acc, e.node, dwl, tlane, c0);

        // Block-level path (Sec. 5.2).  `reaches` : the team's node extends to the end of the wave;
        // `goes_on`: ... and its last group lies behind this wave, in this block.
        const bool reaches = valid && wave_last_node == e.node;
        const bool goes_on = reaches && lastflag == 0 && wave + 1 < nw && g0 + (int64_t)(wave + 1) * G < num_ng;
        const bool waits = leader && !complete_in_wave && goes_on;  // a leader that others hand their parts to
        if (__any(from_prev || waits)) {
            if (from_prev) {
                float *srow = s_slot + (size_t)wave * dim;
#pragma unroll
                for (int c = 0; c < ITER; ++c) {
                    const int d = ((c0 + c) * dwl + tlane) * VEC;
                    if (d < dim) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) srow[d + j] = acc[c][j];
                    }
                }
                if (tlane == 0) {
                    s_last[wave] = lastflag;
                    s_more[wave] = goes_on ? 1 : 0;
                }
            }
            __syncthreads();  // producers and waiting leaders only: every other wave of the block has ended or will
            if (waits) {
                for (int w2 = wave + 1; w2 < nw; ++w2) {
                    const float *srow = s_slot + (size_t)w2 * dim;
#pragma unroll
                    for (int c = 0; c < ITER; ++c) {
                        const int d = ((c0 + c) * dwl + tlane) * VEC;
                        if (d < dim) {
#pragma unroll
                            for (int j = 0; j < VEC; ++j) acc[c][j] = op_combine<OP>(acc[c][j], srow[d + j]);
                        }
                    }
                    block_last |= s_last[w2];
                    if (s_more[w2] == 0) break;
                }
            }
            if (!FULL && c0 + ITER < p.iter_total) __syncthreads();  // the slots are written again in the next pass
        }

        // leader flush (Algorithm 1) of a node that the wave alone did not finish
        if (leader && !complete_in_wave) {
            const bool complete = first && (lastflag | block_last) != 0;  // the block holds all groups of the node
            spans_blocks = !complete;
            // ordered flush: the node of the block's first group goes to partial row 0 of the tile, any other
            // unfinished node (it can only be the node of the last group) to partial row 1
            float *prow = p.part_rows ? p.part_rows + ((size_t)tile * 2 + (team == 0 ? 0 : 1)) * dim : nullptr;
#pragma unroll
            for (int c = 0; c < ITER; ++c) {
                const int d = ((c0 + c) * dwl + tlane) * VEC;
                if (d < dim) {
                    float r[VEC];
                    if (complete) {
                        const float rs = row_scale(p, e.node);
#pragma unroll
                        for (int j = 0; j < VEC; ++j) r[j] = epilogue(acc[c][j] * rs, p.bias, d + j, p.relu);
                        if (p.stream_out) store_vec_stream<VEC>(orow + d, r);
                        else store_vec<VEC>(orow + d, r);
                    } else if (prow) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) r[j] = acc[c][j];
                        store_vec_coherent<VEC>(prow + d, r);
                    } else {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) atomicAdd(&orow[d + j], acc[c][j]);
                    }
                }
            }
        }
    }

    if (spans_blocks && p.part_rows) {
        // The node spans the tiles b0..b1.  Every one of them publishes its partial row (the
        // stores above have completed once the wait below returns), then counts itself in; the
        // block that arrives last adds the partial rows in tile order, applies bias/activation
        // and writes the row, so the result does not depend on timing.
        // (a workgroup-scope fence alone does not wait for the write-through stores: the explicit
        // wait keeps the counter from overtaking them on its way to another memory channel)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        float *orow = p.out + (size_t)e.node * dim;
        int arrived = 0;
        if (tlane == 0) arrived = atomicAdd(&p.cnt[e.node], 1);
        arrived = __shfl(arrived, lane - tlane);
        const int gfirst = p.ngptr[e.node], gend = p.ngptr[e.node + 1];
        const int64_t b0 = gfirst / T, b1 = (gend - 1) / T;
        if (arrived == (int)(b1 - b0)) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            if (tlane == 0) p.cnt[e.node] = 0;  // ready for the next call
            // in its first tile the node is the tile's first node only if it starts the tile
            const float *first_row = p.part_rows + ((size_t)b0 * 2 + (gfirst % T == 0 ? 0 : 1)) * dim;
            for (int c = 0; c < p.iter_total; ++c) {
                const int d = (c * dwl + tlane) * VEC;
                if (d >= dim) break;
                float sum[VEC];
                load_vec_coherent<VEC>(sum, first_row + d);
                for (int64_t b = b0 + 1; b <= b1; b += 4) {
                    float t[4][VEC];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) t[q][j] = op_identity<OP>();
                        if (b + q <= b1) load_vec_coherent<VEC>(t[q], p.part_rows + ((size_t)(b + q) * 2) * dim + d);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (b + q <= b1) {
#pragma unroll
                            for (int j = 0; j < VEC; ++j) sum[j] = op_combine<OP>(sum[j], t[q][j]);
                        }
                }
                const float rs = row_scale(p, e.node);
#pragma unroll
                for (int j = 0; j < VEC; ++j) sum[j] = epilogue(sum[j] * rs, p.bias, d + j, p.relu);
                store_vec<VEC>(orow + d, sum);
            }
        }
    }
}

// Ablation of the block-level optimisations: every neighbor group adds its partial row to global
// memory with atomics; `out` must have been initialised (zero, or the self term) beforehand.
template <bool WEIGHTED>
__global__ __launch_bounds__(256) void k_aggregate_noblock(AggParams p)
{
    const WsHeader *hdr = p.hdr;
    if (!header_ok(hdr, p)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) note_stale(p.hdr, p);
        return;
    }
    const int64_t num_ng = hdr->num_ng;
    const int dwl_log2 = p.dwl_log2, dwl = 1 << dwl_log2;
    const int lane = threadIdx.x & 63;
    const int tlane = lane & (dwl - 1);
    const int64_t team = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> dwl_log2;
    if (team >= num_ng) return;
    const NgEntry e = p.ng[team];
    for (int d = tlane; d < p.dim; d += dwl) {
        float acc = 0.0f;
        for (int k = e.start; k < e.end; ++k) {
            const float x = p.X[(size_t)p.colidx[k] * p.dim + d];
            acc = WEIGHTED ? fmaf(p.ew[k], x, acc) : acc + x;
        }
        atomicAdd(&p.out[(size_t)e.node * p.dim + d], acc);
    }
}

// out = SELF ? self_scale * X : 0 for every row (initialisation of the ablation path).
__global__ __launch_bounds__(256) void k_fill_rows(AggParams p, int self)
{
    const int64_t total = (int64_t)p.n * p.dim;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        p.out[i] = self ? p.self_scale * p.X[i] : 0.0f;
}

__global__ __launch_bounds__(256) void k_epilogue_all(AggParams p)
{
    const int64_t total = (int64_t)p.n * p.dim;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        p.out[i] = epilogue(p.out[i], p.bias, (int)(i % p.dim), p.relu);
}

void launch_agg_init(const AggParams &p, bool self, hipStream_t s)
{
    const int64_t blocks = ((int64_t)p.n + 255) / 256;
    if (self) hipLaunchKernelGGL(k_agg_init<true>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(k_agg_init<false>, dim3((unsigned)blocks), dim3(256), 0, s, p);
}

void launch_agg_epilogue_spanning(const AggParams &p, hipStream_t s)
{
    const int64_t blocks = ((int64_t)p.n + 255) / 256;
    hipLaunchKernelGGL(k_agg_epilogue_spanning, dim3((unsigned)blocks), dim3(256), 0, s, p);
}

template <int VEC, int ITER, int U, int DL, bool FULL>
static void launch_one(int op, bool weighted, bool self, dim3 grid, dim3 block, size_t lds, hipStream_t s,
                       const AggParams &p)
{
    if (p.evec) {
        // half the rows in flight: every neighbour row comes with a row of edge features
        constexpr int UE = U >= 2 ? U / 2 : 1;
        hipLaunchKernelGGL((k_aggregate<VEC, ITER, UE, -1, false, false, kOpSum, false, true>), grid, block, lds, s, p);
    } else if (op == kOpMax) hipLaunchKernelGGL((k_aggregate<VEC, ITER, U, -1, false, false, kOpMax, false>), grid, block, lds, s, p);
    else if (op == kOpMin) hipLaunchKernelGGL((k_aggregate<VEC, ITER, U, -1, false, false, kOpMin, false>), grid, block, lds, s, p);
    else if (self) hipLaunchKernelGGL((k_aggregate<VEC, ITER, U, DL, false, true, kOpSum, FULL>), grid, block, lds, s, p);
    else if (weighted) hipLaunchKernelGGL((k_aggregate<VEC, ITER, U, DL, true, false, kOpSum, FULL>), grid, block, lds, s, p);
    else hipLaunchKernelGGL((k_aggregate<VEC, ITER, U, DL, false, false, kOpSum, FULL>), grid, block, lds, s, p);
}

// The sums over 16-byte loads whose rows are covered in one pass with no idle lane (dim = chunks x team
// width x 4: 16, 32, 64, 96, 128, ... with the model's team width) get the team width as a compile-time
// constant and no bounds checks; everything else takes the generic form.
template <int VEC, int ITER, int U>
static void launch_main(int op, bool weighted, bool self, dim3 grid, dim3 block, size_t lds, hipStream_t s,
                        const AggParams &p)
{
    if constexpr (VEC == 4) {
        if (p.full_rows && op == kOpSum && !p.evec) {
            switch (p.dwl_log2) {
                case 0: launch_one<VEC, ITER, U, 0, true>(op, weighted, self, grid, block, lds, s, p); break;
                case 1: launch_one<VEC, ITER, U, 1, true>(op, weighted, self, grid, block, lds, s, p); break;
                case 2: launch_one<VEC, ITER, U, 2, true>(op, weighted, self, grid, block, lds, s, p); break;
                case 3: launch_one<VEC, ITER, U, 3, true>(op, weighted, self, grid, block, lds, s, p); break;
                case 4: launch_one<VEC, ITER, U, 4, true>(op, weighted, self, grid, block, lds, s, p); break;
                case 5: launch_one<VEC, ITER, U, 5, true>(op, weighted, self, grid, block, lds, s, p); break;
                default: launch_one<VEC, ITER, U, 6, true>(op, weighted, self, grid, block, lds, s, p); break;
            }
            return;
        }
    }
    launch_one<VEC, ITER, U, -1, false>(op, weighted, self, grid, block, lds, s, p);
}

// ---- what the calling thread launched last (gnn_bench_last_aggregation) ----
struct LastLaunch {
    const char *kernel;
    int vec, iter, u, dl, weighted, self, op, T, ngs, wpb, ordered, xcd;
};
static thread_local LastLaunch g_last = {"none", 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

void note_launch(const char *kernel, int vec, int iter, int u, int dl, bool weighted, bool self, int op, int T, int ngs,
                 int wpb, bool ordered, bool xcd)
{
    g_last = LastLaunch{kernel, vec, iter, u, dl, weighted ? 1 : 0, self ? 1 : 0, op, T, ngs, wpb, ordered ? 1 : 0, xcd ? 1 : 0};
}

// U of launch_vec below, for the launch description
static int unroll_of(int vec, int iter)
{
    switch (iter) {
        case 1: return 8;
        case 2: return vec == 4 ? 4 : 8;
        case 3: return 4;
        default: return vec == 4 ? 2 : 4;
    }
}

template <int VEC>
static void launch_vec(int op, int iter, bool weighted, bool self, dim3 grid, dim3 block, size_t lds, hipStream_t s,
                       const AggParams &p)
{
    // U neighbor rows in flight per lane, sized so that U*ITER*VEC stays near 32 registers
    constexpr int U1 = 8, U2 = VEC == 4 ? 4 : 8, U3 = 4, U4 = VEC == 4 ? 2 : 4;
    switch (iter) {
        case 1: launch_main<VEC, 1, U1>(op, weighted, self, grid, block, lds, s, p); break;
        case 2: launch_main<VEC, 2, U2>(op, weighted, self, grid, block, lds, s, p); break;
        case 3: launch_main<VEC, 3, U3>(op, weighted, self, grid, block, lds, s, p); break;
        default: launch_main<VEC, 4, U4>(op, weighted, self, grid, block, lds, s, p); break;
    }
}

// Shared implementation of gnn_aggregate_gcn / gnn_aggregate_gin and of the aggregation step of
// gnn_layer_forward.  self: add self_scale * X[i] (GIN).  bias/relu: fused epilogue.  ws_reserved:
// bytes at the front of the workspace that the caller uses itself (0: only the partition); the
// partial rows of the ordered flush are placed behind them.
int aggregate_reduce_impl(int op, bool mean, bool self, float self_scale, int32_t n, int64_t nnz, const int32_t *rowptr,
                          const int32_t *colidx, const float *ew, const float *X, float *out, int32_t dim, int32_t ngs,
                          int32_t dw, int32_t wpb, uint32_t flags, const float *bias, int relu, void *workspace,
                          size_t workspace_bytes, size_t ws_reserved, hipStream_t s, hipEvent_t ev_start,
                          hipEvent_t ev_stop, FuseSpec *fuse, const float *evec)
{
    const bool plain_sum = op == kOpSum && !mean;
    // per-entry feature vectors: plain sum, no scalar weights, no self term, ordered flush only
    if (evec && (!plain_sum || ew || self || fuse ||
                 (flags & (GNN_FLAG_NO_BLOCK_OPT | GNN_FLAG_ATOMIC_FLUSH | GNN_FLAG_FUSION))))
        return GNN_EINVAL;
    if (op != kOpSum && op != kOpMax && op != kOpMin) return GNN_EINVAL;
    if (!plain_sum && (mean && op != kOpSum)) return GNN_EINVAL;
    if (!plain_sum && (ew || self || fuse)) return GNN_EINVAL;
    if (!plain_sum && (flags & (GNN_FLAG_NO_BLOCK_OPT | GNN_FLAG_ATOMIC_FLUSH | GNN_FLAG_FUSION)))
        return GNN_EINVAL;
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31) || dim <= 0 || ngs < 0 || dw < 0 || wpb < 0) return GNN_EINVAL;
    if (!rowptr || (nnz > 0 && !colidx)) return GNN_EINVAL;
    if (n > 0 && (!X || !out)) return GNN_EINVAL;
    if (X == out && n > 0) return GNN_EINVAL;
    if (dw > 64 || (dw & (dw - 1)) != 0) return GNN_EINVAL;
    if (wpb > kMaxWavesPerBlock) return GNN_EINVAL;
    const bool det = (flags & GNN_FLAG_DETERMINISTIC) != 0;
    const bool atomic_flush = (flags & GNN_FLAG_ATOMIC_FLUSH) != 0;
    if (det && ((flags & GNN_FLAG_NO_BLOCK_OPT) || atomic_flush)) return GNN_EINVAL;
    if (n == 0) return GNN_OK;
    const bool auto_wpb = wpb == 0;

    const int vec = pick_vec(dim, X, out);

    decide_defaults(n, nnz, 0, dim, vec, &ngs, &dw, &wpb);
    int dwl_log2 = 0;
    while ((1 << dwl_log2) < dw) ++dwl_log2;

    const WsLayout L = ws_layout(n, nnz, 0, ngs);
    if (!workspace || ((uintptr_t)workspace) % kAlign != 0 || workspace_bytes < L.total) return GNN_EWORKSPACE;
    char *ws = (char *)workspace;

    if (!(flags & GNN_FLAG_REUSE_PARTITION)) {
        const int rc = partition_build_impl(n, nnz, rowptr, ngs, workspace, workspace_bytes, s);
        if (rc != GNN_OK) return rc;
    }

    AggParams p;
    p.hdr = (WsHeader *)(ws + L.header);
    p.ng = (const NgEntry *)(ws + L.ng);
    p.ngptr = (const int *)(ws + L.ngptr);
    p.colidx = colidx;
    p.ew = ew;
    p.evec = evec;
    p.X = X;
    p.out = out;
    p.part_rows = nullptr;
    p.cnt = (int *)(ws + L.cnt);
    p.bias = bias;
    p.rowptr = mean ? rowptr : nullptr;
    p.self_scale = self_scale;
    p.relu = relu;
    p.n = n;
    p.dim = dim;
    p.ngs = ngs;
    p.dwl_log2 = dwl_log2;
    p.nnz = nnz;
    p.rowptr_key = (uint64_t)(uintptr_t)rowptr;
    // runs of consecutive tiles per XCD: by default from ngs = 16 on (1-3 % faster on all five
    // configurations; with smaller groups it measured up to 15 % slower), always on request
    p.xcd_remap = ((flags & GNN_FLAG_XCD_RUNS) || ngs >= 16) ? 1 : 0;
    p.do_empty = 0;
    // streaming stores only for rows made of whole 128-byte lines: shorter rows share a line with
    // their neighbours and are better merged in L2
    p.stream_out = (dim % 32 == 0) ? 1 : 0;
    p.tile_blocks = 0;
    p.extra_blocks = 0;
    const int units = (dim + vec - 1) / vec;
    p.iter_total = (units + dw - 1) / dw;
    p.plain_rows = (p.stream_out && !bias && !relu && !mean) ? 1 : 0;
    p.full_rows = (p.iter_total <= 4 && p.iter_total * dw * vec == dim) ? 1 : 0;

    const int64_t ng_cap = L.ng_capacity;
    const bool weighted = ew != nullptr;

    if (flags & GNN_FLAG_NO_BLOCK_OPT) {
        p.T = 1;
        hipLaunchKernelGGL(k_fill_rows, dim3(2048), dim3(256), 0, s, p, self ? 1 : 0);
        const int64_t threads = ng_cap << dwl_log2;
        const int64_t blocks = (threads + 255) / 256;
        if (blocks > 0) {
            if (weighted) hipLaunchKernelGGL(k_aggregate_noblock<true>, dim3((unsigned)blocks), dim3(256), 0, s, p);
            else hipLaunchKernelGGL(k_aggregate_noblock<false>, dim3((unsigned)blocks), dim3(256), 0, s, p);
        }
        if (bias || relu) hipLaunchKernelGGL(k_epilogue_all, dim3(2048), dim3(256), 0, s, p);
        note_launch("k_aggregate_noblock", 1, 1, 1, -1, weighted, self, op, 1, ngs, 4, false, false);
        GNN_HIP_TRY(hipGetLastError());
        return GNN_OK;
    }

    // GIN layer with the Update fused in: on request, and by itself for graphs with short rows, where
    // it measured faster than the two separate kernels (one launch per layer, the aggregate never
    // goes to memory).  The caller runs the Update separately if the shape is not covered.
    if (fuse) fuse->done = false;
    const double avg_row = n > 0 ? (double)nnz / (double)n : 0.0;
    const bool kernel_chosen = (flags & GNN_FLAG_XCD_RUNS) != 0;
    // A GCN layer that aggregates first (a widening layer) can be fused the same way, on request only: on the
    // 16 -> 22 layer of a 410 k-node graph the fused kernel took 89 us against 52 + 14 us.
    // (measured: the wave-tile form of the fused layer wins on short rows at every size, -20 % of a model pass
    // on 44 k nodes and on 1.9 M; the block-tile form, which serves the shapes the other does not cover, only
    // while the layer's input stays in the 256 MB memory-side cache)
    const bool small_enough = (double)n * (double)dim * 4.0 <= 160e6;
    const bool wave_tiles_cover = fuse && gin_layer_fused_wave_tiles(p, vec, fuse->M);
    if (fuse && !atomic_flush && !(flags & GNN_FLAG_NO_FUSION) &&
        ((flags & GNN_FLAG_FUSION) || (self && avg_row < 8.0 && (small_enough || wave_tiles_cover) && !kernel_chosen))) {
        // large tiles (up to 64 groups) amortise the copy of W every block makes
        int wpb_f = wpb;
        if (auto_wpb) {
            wpb_f = 8;
            while (wpb_f > 1 && wpb_f * (64 >> dwl_log2) > 64) wpb_f /= 2;
        }
        AggParams pf = p;
        pf.T = wpb_f * (64 >> dwl_log2);
        const bool wave_tiles = wave_tiles_cover;
        if (wave_tiles) {
            pf.T = kFusedWaveTile;
            wpb_f = 8;
        }
        const int32_t part_dim = fuse->M > dim ? fuse->M : dim;  // fused partial rows are M wide
        size_t off = L.total > ws_reserved ? L.total : ws_reserved;
        off = align_up(off);
        if (off + part_rows_bytes(ng_cap, pf.T, part_dim) <= workspace_bytes) {
            pf.part_rows = (float *)(ws + off);
            if (ev_start) GNN_HIP_TRY(hipEventRecord(ev_start, s));
            const int rc = try_gin_layer_fused(pf, vec, wpb_f, fuse->W, fuse->b, fuse->out, fuse->M, fuse->relu,
                                                (ng_cap + pf.T - 1) / pf.T, s, &wpb_f);
            if (rc < 0) return rc;
            if (rc == GNN_OK) {
                const int it_f = p.iter_total < 4 ? p.iter_total : 4;
                note_launch(wave_tiles ? "k_gin_layer_fused_w" : "k_gin_layer_fused", vec, it_f, unroll_of(vec, it_f),
                            wave_tiles ? dwl_log2 : -1, weighted, self, op, pf.T, ngs, wpb_f, true, p.xcd_remap != 0);
                if (ev_stop) GNN_HIP_TRY(hipEventRecord(ev_stop, s));
                fuse->done = true;
                GNN_HIP_TRY(hipGetLastError());
                return GNN_OK;
            }
            // not covered: the taps are recorded again around the aggregation kernel below
        } else if (det) {
            return GNN_EWORKSPACE;
        }
    }

    // the workspace-size functions allow deterministic scratch for blocks of kPartMinTile groups
    if ((det || !plain_sum || evec) && auto_wpb)
        while (wpb * (64 >> dwl_log2) < kPartMinTile && wpb < kMaxWavesPerBlock) wpb *= 2;
    const int T = wpb * (64 >> dwl_log2);
    p.T = T;
    const size_t lds = agg_lds_bytes(T, ngs, dim, wpb, weighted);
    if (lds > kMaxLdsBytes) return GNN_ELIMIT;

    const int64_t tiles_upper = (ng_cap + T - 1) / T;
    const int64_t init_blocks = ((int64_t)n + 255) / 256;
    const int iter = p.iter_total < 4 ? p.iter_total : 4;

    // Ordered flush (one launch, no float atomics, no zeroing pass) whenever the workspace has room
    // for the partial rows behind the caller's own use of it; the atomic flush of Sec. 5.2 otherwise
    // or on request.
    float *part_rows = nullptr;
    {
        size_t off = L.total > ws_reserved ? L.total : ws_reserved;
        off = align_up(off);
        if (off + part_rows_bytes(ng_cap, T, dim) <= workspace_bytes) part_rows = (float *)(ws + off);
    }
    if ((det || !plain_sum || evec) && !part_rows) return GNN_EWORKSPACE;

    const bool ordered = det || evec != nullptr || (part_rows != nullptr && !atomic_flush);

    int64_t grid = tiles_upper;
    if (p.xcd_remap) grid = (tiles_upper + kNumXcd * kXcdRun - 1) / (kNumXcd * kXcdRun) * (kNumXcd * kXcdRun);
    // rows without entries: blocks appended to the grid, each wave taking about four 64-node chunks
    const int64_t nchunks = ((int64_t)n + 63) / 64;
    int64_t extra = (nchunks + (int64_t)wpb * 4 - 1) / ((int64_t)wpb * 4);
    if (extra > 8192) extra = 8192;
    extra = (extra + kNumXcd - 1) / kNumXcd * kNumXcd;
    p.do_empty = 1;
    p.tile_blocks = grid;
    p.extra_blocks = (int)extra;
    if (grid + extra >= ((int64_t)1 << 31)) return GNN_ELIMIT;

    // (the ordered flush adds nothing to `out`, so no row needs zeroing and no pass follows)
    if (ordered) p.part_rows = part_rows;
    else if (self) hipLaunchKernelGGL(k_agg_init<true>, dim3((unsigned)init_blocks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(k_agg_init<false>, dim3((unsigned)init_blocks), dim3(256), 0, s, p);

    if (ev_start) GNN_HIP_TRY(hipEventRecord(ev_start, s));
    {
        const dim3 g((unsigned)(grid + extra)), b((unsigned)(wpb * 64));
        if (vec == 4) launch_vec<4>(op, iter, weighted, self, g, b, lds, s, p);
        else if (vec == 2) launch_vec<2>(op, iter, weighted, self, g, b, lds, s, p);
        else launch_vec<1>(op, iter, weighted, self, g, b, lds, s, p);
    }
    if (evec) {
        const int u = unroll_of(vec, iter);
        note_launch("k_aggregate(edge vectors)", vec, iter, u >= 2 ? u / 2 : 1, -1, false, false, op, T, ngs, wpb, ordered, p.xcd_remap != 0);
    } else
    note_launch("k_aggregate", vec, iter, unroll_of(vec, iter), (vec == 4 && op == kOpSum && p.full_rows) ? dwl_log2 : -1,
                weighted && op == kOpSum, self && op == kOpSum, op, T, ngs,
                wpb, ordered, p.xcd_remap != 0);
    if (ev_stop) GNN_HIP_TRY(hipEventRecord(ev_stop, s));
    if (!ordered && (bias || relu))
        hipLaunchKernelGGL(k_agg_epilogue_spanning, dim3((unsigned)init_blocks), dim3(256), 0, s, p);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

// ---- scratch memory of gnn_aggregate_gin_static: one array per GPU, held until the process ends ----
constexpr size_t kStaticScratchBytes = (size_t)128 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, looked up once per GPU

// Device address of the current GPU's copy of `scratch` (in host code the array's name is only a
// stand-in: it must never be passed to a kernel or a memset).
static int static_scratch(void **ptr)
{
    int dev = 0;
    GNN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return GNN_ELIMIT;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        GNN_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return GNN_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" {

int gnn_bench_last_aggregation(char *buf, size_t cap)
{
    if (!buf || cap == 0) return GNN_EINVAL;
    const LastLaunch &l = g_last;
    const int k = snprintf(buf, cap, "%s<%d,%d,%d,%d,%s,%s,%d> groups/block=%d ngs=%d waves/block=%d flush=%s tiles=%s",
                           l.kernel, l.vec, l.iter, l.u, l.dl, l.weighted ? "true" : "false", l.self ? "true" : "false",
                           l.op, l.T, l.ngs, l.wpb, l.ordered ? "ordered" : "atomic", l.xcd ? "xcd-runs" : "round-robin");
    return (k < 0 || (size_t)k >= cap) ? GNN_ELIMIT : GNN_OK;
}

int gnn_aggregate_gin_static(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float eps,
                             const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw, int32_t waves_per_block,
                             uint32_t flags, void *stream, void **scratch_out)
{
    if (n < 0 || nnz < 0 || dim <= 0 || ngs < 0) return GNN_EINVAL;
    // the same layout gnn_workspace_bytes sizes for max_dim = dim (room for the ordered flush), with the
    // group size the call will use
    int32_t r_ngs = ngs, r_dw = dw > 0 && dw <= 64 && (dw & (dw - 1)) == 0 ? dw : 0, r_wpb = 0;
    decide_defaults(n, nnz, 0, dim, 1, &r_ngs, &r_dw, &r_wpb);
    const WsLayout L = ws_layout(n, nnz, 0, r_ngs);
    const size_t need = L.total + part_rows_bytes(L.ng_capacity, kPartMinTile, dim);
    if (need > kStaticScratchBytes) return GNN_ELIMIT;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != GNN_OK) return rc;
    if (scratch_out) *scratch_out = ws;
    return aggregate_impl(true, 1.0f + eps, n, nnz, rowptr, colidx, nullptr, X, out, dim, ngs, dw, waves_per_block,
                          flags, nullptr, 0, ws, kStaticScratchBytes, 0, (hipStream_t)stream, nullptr, nullptr,
                          nullptr);
}

int gnn_aggregate_gcn(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *ew,
                      const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw, int32_t waves_per_block,
                      uint32_t flags, void *workspace, size_t workspace_bytes, void *stream)
{
    return aggregate_impl(false, 0.0f, n, nnz, rowptr, colidx, ew, X, out, dim, ngs, dw, waves_per_block, flags,
                          nullptr, 0, workspace, workspace_bytes, 0, (hipStream_t)stream, nullptr, nullptr, nullptr);
}

int gnn_aggregate_gin(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float eps,
                      const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw, int32_t waves_per_block,
                      uint32_t flags, void *workspace, size_t workspace_bytes, void *stream)
{
    return aggregate_impl(true, 1.0f + eps, n, nnz, rowptr, colidx, nullptr, X, out, dim, ngs, dw, waves_per_block,
                          flags, nullptr, 0, workspace, workspace_bytes, 0, (hipStream_t)stream, nullptr, nullptr,
                          nullptr);
}

int gnn_aggregate_reduce(int op, int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *X,
                         float *out, int32_t dim, int32_t ngs, int32_t dw, int32_t waves_per_block, uint32_t flags,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    int kop = kOpSum;
    bool mean = false;
    switch (op) {
        case GNN_REDUCE_SUM: break;
        case GNN_REDUCE_MAX: kop = kOpMax; break;
        case GNN_REDUCE_MIN: kop = kOpMin; break;
        case GNN_REDUCE_MEAN: mean = true; break;
        default: return GNN_EINVAL;
    }
    return aggregate_reduce_impl(kop, mean, false, 0.0f, n, nnz, rowptr, colidx, nullptr, X, out, dim, ngs, dw,
                                 waves_per_block, flags, nullptr, 0, workspace, workspace_bytes, 0, (hipStream_t)stream,
                                 nullptr, nullptr, nullptr);
}

int gnn_aggregate_edge(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *E,
                       const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw, int32_t waves_per_block,
                       uint32_t flags, void *workspace, size_t workspace_bytes, void *stream)
{
    if (nnz > 0 && !E) return GNN_EINVAL;
    if (nnz == 0) E = nullptr;
    // (a graph without entries: every row is 0, which the plain sum writes)
    return aggregate_reduce_impl(kOpSum, false, false, 0.0f, n, nnz, rowptr, colidx, nullptr, X, out, dim, ngs, dw,
                                 waves_per_block, flags, nullptr, 0, workspace, workspace_bytes, 0, (hipStream_t)stream,
                                 nullptr, nullptr, nullptr, E);
}

}  // extern "C"
