// Graph preparation on the device: a round-based, data-parallel schedule of the community
// renumbering of Sec. 5.1, the CSR relabelling that applies a permutation, and the GCN weights of
// Eq. 2.  One-time work per graph: these calls allocate their own temporaries and synchronise.
//
// Renumbering.  Sec. 5.1 asks for ids that follow communities found by merging for modularity and
// leaves the merge schedule open.  The host version (gnn_reorder) merges one vertex at a time; here
// all communities act on the same state in synchronous rounds, which maps onto sorts, scans and
// per-edge kernels:
//   1. per edge (u, v, w) between communities: S = w * M2 - degw(u) * degw(v) (modularity gain up to a
//      positive factor); every community proposes to its neighbour of largest S, smallest id among
//      equals, if S > 0 (an atomic max over the edges, then an atomic min over the edges that reach it);
//   2. of two communities that propose to each other the smaller id stays;
//   3. a proposal u -> t is carried out only if t itself does not move (stars), the rest try again;
//   4. the joiners of t are appended to t's node order by ascending id (sort by (t, id), segmented
//      scan of their sizes); edges are renamed, self edges dropped, parallel edges summed (sort +
//      reduce by key).
// Ends when a round merges nothing.  New ids: communities by ascending root id, nodes by their
// position inside the community.  Everything is integer arithmetic, so the result is reproducible
// bit for bit.  The device-wide sort / scan / reduce-by-key / unique steps are hipCUB's.
#include <hip/hip_runtime.h>
#include <hipcub/hipcub.hpp>

#include <cmath>
#include <vector>

#include "gnn_internal.h"

namespace gnn {

namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(int64_t items)
{
    int64_t b = (items + kThreads - 1) / kThreads;
    if (b < 1) b = 1;
    if (b > 1048576) b = 1048576;  // the kernels below walk with a grid stride
    return (unsigned)b;
}

#define GRID_STRIDE(i, count) \
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < (count); i += (int64_t)gridDim.x * blockDim.x)

__device__ __forceinline__ uint64_t make_key(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

// row that holds entry e: the last i with rowptr[i] <= e
__device__ __forceinline__ int row_of(const int *__restrict__ rowptr, int n, int64_t e)
{
    int lo = 0, hi = n;  // rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if ((int64_t)rowptr[mid] <= e) lo = mid;
        else hi = mid;
    }
    return lo;
}

// ---- initial clean edge list -------------------------------------------------------------------
__global__ void k_edge_keys(int n, int64_t nnz, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                            uint64_t *__restrict__ key, int *__restrict__ counters)
{
    GRID_STRIDE(e, nnz) {
        const int i = row_of(rowptr, n, e), j = colidx[e];
        const bool outside = j < 0 || j >= n;  // malformed CSR: reported, the entry is dropped
        const bool loop = i == j || outside;
        key[e] = loop ? make_key((uint32_t)n, 0u) : make_key((uint32_t)i, (uint32_t)j);
        // flags, not counts: millions of atomics on one address would serialise
        if (loop) counters[0] = 1;
        if (outside) counters[3] = 1;
    }
}

__global__ void k_fill_i32(int *__restrict__ a, int64_t count, int value) { GRID_STRIDE(i, count) a[i] = value; }
__global__ void k_iota_i32(int *__restrict__ a, int64_t count) { GRID_STRIDE(i, count) a[i] = (int)i; }

// clean degree of every node = length of its run in the sorted key list (no atomics: hubs would
// serialise them).  First the run heads note where they start, then the run tails write the length.
__global__ void k_degree_heads(const uint64_t *__restrict__ key, int64_t m, int *__restrict__ run_start)
{
    GRID_STRIDE(e, m) {
        const int cu = (int)(key[e] >> 32);
        if (e == 0 || (int)(key[e - 1] >> 32) != cu) run_start[cu] = (int)e;
    }
}

__global__ void k_degree_tails(const uint64_t *__restrict__ key, int64_t m, const int *__restrict__ run_start,
                               int *__restrict__ degw)
{
    GRID_STRIDE(e, m) {
        const int cu = (int)(key[e] >> 32);
        if (e == m - 1 || (int)(key[e + 1] >> 32) != cu) degw[cu] = (int)e + 1 - run_start[cu];
    }
}

// ---- one round ---------------------------------------------------------------------------------
__global__ void k_round_init(int n, long long *__restrict__ bestS, int *__restrict__ bestv, int *__restrict__ shift,
                             int *__restrict__ counters)
{
    GRID_STRIDE(u, n) {
        bestS[u] = LLONG_MIN;
        bestv[u] = INT_MAX;
        shift[u] = 0;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) counters[1] = counters[2] = 0;
}

__device__ __forceinline__ long long edge_score(uint64_t k, int w, long long M2, const int *__restrict__ degw)
{
    const int cu = (int)(k >> 32), cv = (int)(uint32_t)k;
    return (long long)w * M2 - (long long)degw[cu] * (long long)degw[cv];
}

__global__ void k_score_max(const uint64_t *__restrict__ key, const int *__restrict__ w, int64_t m, long long M2,
                            const int *__restrict__ degw, long long *__restrict__ bestS)
{
    // The keys are sorted, so the edges of one community are neighbours: the lanes of a wave first
    // combine the scores of equal communities among themselves (segmented max scan over the wave),
    // and only the last lane of every run goes to memory -- a hub's 10^4 edges cost 10^2 atomics.
    const int lane = threadIdx.x & 63;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t base = (int64_t)blockIdx.x * blockDim.x + threadIdx.x - lane; base < m; base += stride) {
        const int64_t e = base + lane;
        const bool live = e < m;
        const int cu = live ? (int)(key[e] >> 32) : -1;
        long long sc = live ? edge_score(key[e], w[e], M2, degw) : LLONG_MIN;
        for (int o = 1; o < 64; o <<= 1) {
            const int ocu = __shfl_up(cu, o);
            const long long osc = __shfl_up(sc, o);
            if (lane >= o && ocu == cu && osc > sc) sc = osc;
        }
        const int ncu = __shfl_down(cu, 1);
        if (live && (lane == 63 || ncu != cu)) atomicMax(&bestS[cu], sc);
    }
}

__global__ void k_score_arg(const uint64_t *__restrict__ key, const int *__restrict__ w, int64_t m, long long M2,
                            const int *__restrict__ degw, const long long *__restrict__ bestS, int *__restrict__ bestv)
{
    GRID_STRIDE(e, m) {
        const int cu = (int)(key[e] >> 32);
        if (edge_score(key[e], w[e], M2, degw) == bestS[cu]) atomicMin(&bestv[cu], (int)(uint32_t)key[e]);
    }
}

__global__ void k_best(int n, const long long *__restrict__ bestS, const int *__restrict__ bestv, int *__restrict__ best)
{
    GRID_STRIDE(u, n) best[u] = (bestS[u] > 0 && bestv[u] != INT_MAX) ? bestv[u] : (int)u;
}

__global__ void k_mutual(int n, const int *__restrict__ best, int *__restrict__ prop)
{
    GRID_STRIDE(u, n) {
        const int b = best[u];
        prop[u] = (b != (int)u && best[b] == (int)u && (int)u < b) ? (int)u : b;
    }
}

// target[u] = where u goes this round (itself if it stays); joiners get the sort key (target, id)
__global__ void k_stars(int n, const int *__restrict__ prop, const int *__restrict__ size, int *__restrict__ target,
                        uint64_t *__restrict__ jkey, int *__restrict__ jsize, int *__restrict__ counters)
{
    GRID_STRIDE(u, n) {
        const int p = prop[u];
        const bool joins = p != (int)u && prop[p] == p;
        target[u] = joins ? p : (int)u;
        jkey[u] = joins ? make_key((uint32_t)p, (uint32_t)u) : make_key((uint32_t)n, 0u);
        jsize[u] = joins ? size[u] : 0;
        // number of joiners: one atomic per wave
        const unsigned long long votes = __ballot(joins);
        if (votes != 0ull && (threadIdx.x & 63) == (unsigned)(__ffsll((long long)votes) - 1))
            atomicAdd(&counters[1], __popcll(votes));
    }
}

__global__ void k_group_heads(const uint64_t *__restrict__ jkey, const int *__restrict__ before, int64_t count,
                              int *__restrict__ head)
{
    GRID_STRIDE(k, count) {
        const bool first = k == 0 || (jkey[k] >> 32) != (jkey[k - 1] >> 32);
        head[k] = first ? before[k] : 0;
    }
}

__global__ void k_shift(const uint64_t *__restrict__ jkey, const int *__restrict__ before, const int *__restrict__ start,
                        int64_t count, const int *__restrict__ size, int *__restrict__ shift)
{
    GRID_STRIDE(k, count) {
        const int t = (int)(jkey[k] >> 32), j = (int)(uint32_t)jkey[k];
        shift[j] = size[t] + before[k] - start[k];
    }
}

__global__ void k_move_nodes(int n, const int *__restrict__ shift, const int *__restrict__ target, int *__restrict__ comm,
                             int *__restrict__ pos)
{
    GRID_STRIDE(v, n) {
        const int c = comm[v];
        pos[v] += shift[c];
        comm[v] = target[c];
    }
}

__global__ void k_grow_targets(const uint64_t *__restrict__ jkey, const int *__restrict__ jsize, int64_t count,
                               int *__restrict__ size, int *__restrict__ degw)
{
    GRID_STRIDE(k, count) {
        const int t = (int)(jkey[k] >> 32), j = (int)(uint32_t)jkey[k];
        atomicAdd(&size[t], jsize[k]);
        atomicAdd(&degw[t], degw[j]);  // a joiner is nobody's target in the same round: degw[j] is stable
    }
}

__global__ void k_rename_edges(int n, uint64_t *__restrict__ key, int64_t m, const int *__restrict__ target,
                               int *__restrict__ counters)
{
    GRID_STRIDE(e, m) {
        const int cu = target[(int)(key[e] >> 32)], cv = target[(int)(uint32_t)key[e]];
        const bool inner = cu == cv;
        key[e] = inner ? make_key((uint32_t)n, 0u) : make_key((uint32_t)cu, (uint32_t)cv);
        if (inner) counters[2] = 1;  // a flag: some edge fell inside a community
    }
}

// ---- final numbering ---------------------------------------------------------------------------
__global__ void k_root_sizes(int n, const int *__restrict__ comm, const int *__restrict__ size, int *__restrict__ rs)
{
    GRID_STRIDE(v, n) rs[v] = comm[v] == (int)v ? size[v] : 0;
}

__global__ void k_number(int n, const int *__restrict__ comm, const int *__restrict__ pos, const int *__restrict__ base,
                         int *__restrict__ perm, int *__restrict__ iperm)
{
    GRID_STRIDE(v, n) {
        const int p = base[comm[v]] + pos[v];
        perm[v] = p;
        iperm[p] = (int)v;
    }
}

// ---- relabelling and weights -------------------------------------------------------------------
__global__ void k_relabel_keys(int n, int64_t nnz, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                               const int *__restrict__ perm, uint64_t *__restrict__ key, int *__restrict__ entry,
                               int *__restrict__ bad)
{
    GRID_STRIDE(e, nnz) {
        const int i = row_of(rowptr, n, e);
        int j = colidx[e];
        if (j < 0 || j >= n) {  // malformed CSR: reported by the caller
            atomicAdd(bad, 1);
            j = 0;
        }
        key[e] = make_key((uint32_t)perm[i], (uint32_t)perm[j]);
        entry[e] = (int)e;
    }
}

__global__ void k_new_lengths(int n, const int *__restrict__ rowptr, const int *__restrict__ perm, int *__restrict__ len2)
{
    GRID_STRIDE(i, n) len2[perm[i]] = rowptr[i + 1] - rowptr[i];
    if (blockIdx.x == 0 && threadIdx.x == 0) len2[n] = 0;
}

__global__ void k_relabel_out(int64_t nnz, const uint64_t *__restrict__ key, const int *__restrict__ entry,
                              const float *__restrict__ val, int *__restrict__ colidx2, float *__restrict__ val2)
{
    GRID_STRIDE(k, nnz) {
        colidx2[k] = (int)(uint32_t)key[k];
        if (val) val2[k] = val[entry[k]];
    }
}

__global__ void k_perm_check(int n, const int *__restrict__ perm, int *__restrict__ seen, int *__restrict__ bad)
{
    GRID_STRIDE(i, n) {
        const int p = perm[i];
        if (p < 0 || p >= n || atomicAdd(&seen[p], 1) != 0) atomicAdd(bad, 1);
    }
}

// Transpose: entry e = (i, j) gets the sort key (j, i); the sorted order is the transposed CSR.
__global__ void k_transpose_keys(int n, int64_t nnz, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                                 uint64_t *__restrict__ key, int *__restrict__ entry, int *__restrict__ len_t,
                                 int *__restrict__ bad)
{
    GRID_STRIDE(e, nnz) {
        const int i = row_of(rowptr, n, e);
        int j = colidx[e];
        if (j < 0 || j >= n) {  // malformed CSR: reported by the caller
            *bad = 1;
            j = 0;
        } else {
            atomicAdd(&len_t[j], 1);
        }
        key[e] = make_key((uint32_t)j, (uint32_t)i);
        entry[e] = (int)e;
    }
}

__global__ void k_transpose_out(int64_t nnz, const uint64_t *__restrict__ key, const int *__restrict__ entry,
                                const float *__restrict__ val, int *__restrict__ colidx_t, float *__restrict__ val_t)
{
    GRID_STRIDE(k, nnz) {
        colidx_t[k] = (int)(uint32_t)key[k];
        if (val) val_t[k] = val[entry[k]];
    }
}

// Eq. 4: sum over the stored entries of |row - column|, one atomic per wave.
__global__ void k_aes_sum(int n, int64_t nnz, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                          unsigned long long *__restrict__ total)
{
    unsigned long long mine = 0;
    GRID_STRIDE(e, nnz) {
        const long long d = (long long)row_of(rowptr, n, e) - (long long)colidx[e];
        mine += (unsigned long long)(d < 0 ? -d : d);
    }
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_down(mine, o);
    if ((threadIdx.x & 63) == 0 && mine != 0ull) atomicAdd(total, mine);
}

__global__ void k_gcn_norm(int n, int64_t nnz, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                           float *__restrict__ ew)
{
    GRID_STRIDE(e, nnz) {
        const int i = row_of(rowptr, n, e), j = colidx[e];
        if (j < 0 || j >= n) {  // malformed CSR (gnn_validate_csr_device reports it)
            ew[e] = 0.0f;
            continue;
        }
        const double di = (double)(rowptr[i + 1] - rowptr[i]), dj = (double)(rowptr[j + 1] - rowptr[j]);
        ew[e] = (float)(1.0 / sqrt(di * dj));
    }
}

// Device temporaries of one call: sizes are registered first, then one allocation serves them all
// (two dozen separate allocations cost more than the kernels of a renumbering), released on return.
struct Arena {
    struct Slot {
        void **out;
        size_t offset;
    };
    std::vector<Slot> slots;
    size_t total = 0;
    char *base = nullptr;
    ~Arena()
    {
        if (base) (void)hipFree(base);
    }
    template <typename T>
    void want(T **out, size_t count)
    {
        slots.push_back({reinterpret_cast<void **>(out), total});
        total += align_up((count > 0 ? count : 1) * sizeof(T));
    }
    int commit()
    {
        void *p = nullptr;
        const hipError_t e = hipMalloc(&p, total > 0 ? total : kAlign);
        if (e != hipSuccess) {
            set_last_hip_error((int)e);
            return GNN_EHIP;
        }
        base = (char *)p;
        for (const Slot &sl : slots) *sl.out = base + sl.offset;
        return GNN_OK;
    }
};

#define GNN_TRY(expr)               \
    do {                            \
        const int rc__ = (expr);    \
        if (rc__ != GNN_OK) return rc__; \
    } while (0)

inline int bit_length(uint32_t x)
{
    int b = 0;
    while (x) {
        ++b;
        x >>= 1;
    }
    return b;
}

}  // namespace

}  // namespace gnn

using namespace gnn;

extern "C" {

int gnn_reorder_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, int32_t *perm,
                       int32_t *iperm, int32_t max_rounds, int32_t *rounds_out, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31) || max_rounds < 0) return GNN_EINVAL;
    if (rounds_out) *rounds_out = 0;
    if (n == 0) return GNN_OK;
    if (!rowptr || !perm || !iperm || (nnz > 0 && !colidx)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int key_bits = 32 + bit_length((uint32_t)n);  // the sentinel (n, 0) sorts last

    Arena mem;
    uint64_t *keyA, *keyB, *jkeyA, *jkeyB;
    int *wA, *wB, *jsA, *jsB, *comm, *pos, *size, *degw, *bestv, *best, *prop, *target, *shift, *before, *head, *start;
    int *counters, *nruns;
    long long *bestS;
    mem.want(&keyA, (size_t)nnz);
    mem.want(&keyB, (size_t)nnz);
    mem.want(&wA, (size_t)nnz);
    mem.want(&wB, (size_t)nnz);
    mem.want(&jkeyA, (size_t)n);
    mem.want(&jkeyB, (size_t)n);
    mem.want(&jsA, (size_t)n);
    mem.want(&jsB, (size_t)n);
    mem.want(&comm, (size_t)n);
    mem.want(&pos, (size_t)n);
    mem.want(&size, (size_t)n);
    mem.want(&degw, (size_t)n);
    mem.want(&bestv, (size_t)n);
    mem.want(&best, (size_t)n);
    mem.want(&prop, (size_t)n);
    mem.want(&target, (size_t)n);
    mem.want(&shift, (size_t)n);
    mem.want(&before, (size_t)n);
    mem.want(&head, (size_t)n);
    mem.want(&start, (size_t)n);
    mem.want(&bestS, (size_t)n);
    mem.want(&counters, 4);
    mem.want(&nruns, 1);

    // temporary storage of the library primitives: the largest any call below asks for (a size query
    // only looks at the types of its pointer arguments)
    size_t tmp_bytes = 0;
    {
        size_t b = 0;
        const int mm = (int)nnz;
        uint64_t *k0 = nullptr, *k1 = nullptr;
        int *v0 = nullptr, *v1 = nullptr, *cnt = nullptr;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortKeys(nullptr, b, k0, k1, mm, 0, key_bits, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, b, k0, k1, v0, v1, mm, 0, key_bits, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceSelect::Unique(nullptr, b, k0, k1, cnt, mm, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceReduce::ReduceByKey(nullptr, b, k0, k1, v0, v1, cnt, hipcub::Sum(), mm, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, b, k0, k1, v0, v1, n, 0, key_bits, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, b, v0, v1, n, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceScan::InclusiveScan(nullptr, b, v0, v1, hipcub::Max(), n, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
    }
    char *tmp;
    mem.want(&tmp, tmp_bytes);
    GNN_TRY(mem.commit());

    int host_counters[4] = {0, 0, 0, 0};
    int host_runs = 0;

    // clean graph: no self loops, duplicate entries once
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(kThreads), 0, s, counters, (int64_t)4, 0);
    hipLaunchKernelGGL(k_iota_i32, dim3(blocks_for(n)), dim3(kThreads), 0, s, comm, (int64_t)n);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n)), dim3(kThreads), 0, s, pos, (int64_t)n, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n)), dim3(kThreads), 0, s, size, (int64_t)n, 1);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n)), dim3(kThreads), 0, s, degw, (int64_t)n, 0);
    int64_t m = 0;
    if (nnz > 0) {
        hipLaunchKernelGGL(k_edge_keys, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, n, nnz, rowptr, colidx, keyA, counters);
        size_t b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortKeys(tmp, b, keyA, keyB, (int)nnz, 0, key_bits, s));
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceSelect::Unique(tmp, b, keyB, keyA, nruns, (int)nnz, s));
        GNN_HIP_TRY(hipMemcpyAsync(host_counters, counters, sizeof(host_counters), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipMemcpyAsync(&host_runs, nruns, sizeof(int), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipStreamSynchronize(s));
        if (host_counters[3] != 0) return GNN_ECSR;
        m = (int64_t)host_runs - (host_counters[0] > 0 ? 1 : 0);  // the self loops collapsed into one last key
        if (m > 0) {
            hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(m)), dim3(kThreads), 0, s, wA, m, 1);
            hipLaunchKernelGGL(k_degree_heads, dim3(blocks_for(m)), dim3(kThreads), 0, s, keyA, m, head);
            hipLaunchKernelGGL(k_degree_tails, dim3(blocks_for(m)), dim3(kThreads), 0, s, keyA, m, head, degw);
        }
    }
    const long long M2 = (long long)m;

    int rounds = 0;
    for (int r = 0; r < max_rounds && m > 0; ++r) {
        const unsigned gn = blocks_for(n), gm = blocks_for(m);
        hipLaunchKernelGGL(k_round_init, dim3(gn), dim3(kThreads), 0, s, n, bestS, bestv, shift, counters);
        hipLaunchKernelGGL(k_score_max, dim3(gm), dim3(kThreads), 0, s, keyA, wA, m, M2, degw, bestS);
        hipLaunchKernelGGL(k_score_arg, dim3(gm), dim3(kThreads), 0, s, keyA, wA, m, M2, degw, bestS, bestv);
        hipLaunchKernelGGL(k_best, dim3(gn), dim3(kThreads), 0, s, n, bestS, bestv, best);
        hipLaunchKernelGGL(k_mutual, dim3(gn), dim3(kThreads), 0, s, n, best, prop);
        hipLaunchKernelGGL(k_stars, dim3(gn), dim3(kThreads), 0, s, n, prop, size, target, jkeyA, jsA, counters);
        GNN_HIP_TRY(hipMemcpyAsync(host_counters, counters, sizeof(host_counters), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipStreamSynchronize(s));
        const int64_t njoin = host_counters[1];
        if (njoin == 0) break;
        ++rounds;
        // joiners by (target, id); their positions behind the target's nodes
        size_t b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(tmp, b, jkeyA, jkeyB, jsA, jsB, n, 0, key_bits, s));
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(tmp, b, jsB, before, (int)njoin, s));
        hipLaunchKernelGGL(k_group_heads, dim3(blocks_for(njoin)), dim3(kThreads), 0, s, jkeyB, before, njoin, head);
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceScan::InclusiveScan(tmp, b, head, start, hipcub::Max(), (int)njoin, s));
        hipLaunchKernelGGL(k_shift, dim3(blocks_for(njoin)), dim3(kThreads), 0, s, jkeyB, before, start, njoin, size, shift);
        hipLaunchKernelGGL(k_move_nodes, dim3(gn), dim3(kThreads), 0, s, n, shift, target, comm, pos);
        hipLaunchKernelGGL(k_grow_targets, dim3(blocks_for(njoin)), dim3(kThreads), 0, s, jkeyB, jsB, njoin, size, degw);
        // edges between the new communities
        hipLaunchKernelGGL(k_rename_edges, dim3(gm), dim3(kThreads), 0, s, n, keyA, m, target, counters);
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(tmp, b, keyA, keyB, wA, wB, (int)m, 0, key_bits, s));
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceReduce::ReduceByKey(tmp, b, keyB, keyA, wB, wA, nruns, hipcub::Sum(), (int)m, s));
        GNN_HIP_TRY(hipMemcpyAsync(host_counters, counters, sizeof(host_counters), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipMemcpyAsync(&host_runs, nruns, sizeof(int), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipStreamSynchronize(s));
        m = (int64_t)host_runs - (host_counters[2] > 0 ? 1 : 0);
    }

    // communities by ascending root id, nodes by position
    {
        const unsigned gn = blocks_for(n);
        hipLaunchKernelGGL(k_root_sizes, dim3(gn), dim3(kThreads), 0, s, n, comm, size, head);
        size_t b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(tmp, b, head, start, n, s));
        hipLaunchKernelGGL(k_number, dim3(gn), dim3(kThreads), 0, s, n, comm, pos, start, perm, iperm);
    }
    GNN_HIP_TRY(hipGetLastError());
    GNN_HIP_TRY(hipStreamSynchronize(s));
    if (rounds_out) *rounds_out = rounds;
    return GNN_OK;
}

int gnn_apply_perm_csr_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                              const int32_t *perm, int32_t *rowptr2, int32_t *colidx2, float *val2, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) return GNN_EINVAL;
    if (!rowptr || !rowptr2 || (n > 0 && !perm) || (val && !val2)) return GNN_EINVAL;
    if (nnz > 0 && (!colidx || !colidx2)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    Arena mem;
    uint64_t *keyA, *keyB;
    int *entA, *entB, *len2, *seen, *bad;
    mem.want(&keyA, (size_t)nnz);
    mem.want(&keyB, (size_t)nnz);
    mem.want(&entA, (size_t)nnz);
    mem.want(&entB, (size_t)nnz);
    mem.want(&len2, (size_t)n + 1);
    mem.want(&seen, (size_t)n + 1);
    mem.want(&bad, 1);
    const int key_bits = 32 + bit_length((uint32_t)n);
    size_t tmp_bytes = 0, b = 0;
    {
        uint64_t *k0 = nullptr, *k1 = nullptr;
        int *v0 = nullptr, *v1 = nullptr;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, b, k0, k1, v0, v1, (int)nnz, 0, key_bits, s));
        tmp_bytes = b;
        GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, b, v0, v1, n + 1, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
    }
    char *tmp;
    mem.want(&tmp, tmp_bytes);
    GNN_TRY(mem.commit());

    // perm must be a bijection of [0, n)
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n + 1)), dim3(kThreads), 0, s, seen, (int64_t)n + 1, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(kThreads), 0, s, bad, (int64_t)1, 0);
    if (n > 0) hipLaunchKernelGGL(k_perm_check, dim3(blocks_for(n)), dim3(kThreads), 0, s, n, perm, seen, bad);
    int host_bad = 0;
    GNN_HIP_TRY(hipMemcpyAsync(&host_bad, bad, sizeof(int), hipMemcpyDeviceToHost, s));
    GNN_HIP_TRY(hipStreamSynchronize(s));
    if (host_bad != 0) return GNN_EINVAL;

    hipLaunchKernelGGL(k_new_lengths, dim3(blocks_for(n)), dim3(kThreads), 0, s, n, rowptr, perm, len2);
    b = tmp_bytes;
    GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(tmp, b, len2, rowptr2, n + 1, s));
    if (nnz > 0) {
        // a stable sort by (new row, new column): equal keys keep the order of their old positions
        hipLaunchKernelGGL(k_relabel_keys, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, n, nnz, rowptr, colidx, perm, keyA, entA,
                           bad);
        GNN_HIP_TRY(hipMemcpyAsync(&host_bad, bad, sizeof(int), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipStreamSynchronize(s));
        if (host_bad != 0) return GNN_ECSR;
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(tmp, b, keyA, keyB, entA, entB, (int)nnz, 0, key_bits, s));
        hipLaunchKernelGGL(k_relabel_out, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, nnz, keyB, entB, val, colidx2, val2);
    }
    GNN_HIP_TRY(hipGetLastError());
    GNN_HIP_TRY(hipStreamSynchronize(s));
    return GNN_OK;
}

int gnn_csr_transpose_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                             int32_t *rowptr_t, int32_t *colidx_t, float *val_t, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) return GNN_EINVAL;
    if (!rowptr || !rowptr_t || (val && !val_t)) return GNN_EINVAL;
    if (nnz > 0 && (!colidx || !colidx_t)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    Arena mem;
    uint64_t *keyA, *keyB;
    int *entA, *entB, *len_t, *bad;
    mem.want(&keyA, (size_t)nnz);
    mem.want(&keyB, (size_t)nnz);
    mem.want(&entA, (size_t)nnz);
    mem.want(&entB, (size_t)nnz);
    mem.want(&len_t, (size_t)n + 1);
    mem.want(&bad, 1);
    const int key_bits = 32 + bit_length((uint32_t)n);
    size_t tmp_bytes = 0, b = 0;
    {
        uint64_t *k0 = nullptr, *k1 = nullptr;
        int *v0 = nullptr, *v1 = nullptr;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, b, k0, k1, v0, v1, (int)nnz, 0, key_bits, s));
        tmp_bytes = b;
        GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, b, v0, v1, n + 1, s));
        tmp_bytes = b > tmp_bytes ? b : tmp_bytes;
    }
    char *tmp;
    mem.want(&tmp, tmp_bytes);
    GNN_TRY(mem.commit());

    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n + 1)), dim3(kThreads), 0, s, len_t, (int64_t)n + 1, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(kThreads), 0, s, bad, (int64_t)1, 0);
    if (nnz > 0)
        hipLaunchKernelGGL(k_transpose_keys, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, n, nnz, rowptr, colidx, keyA, entA,
                           len_t, bad);
    int host_bad = 0;
    GNN_HIP_TRY(hipMemcpyAsync(&host_bad, bad, sizeof(int), hipMemcpyDeviceToHost, s));
    GNN_HIP_TRY(hipStreamSynchronize(s));
    if (host_bad != 0) return GNN_ECSR;
    b = tmp_bytes;
    GNN_HIP_TRY(hipcub::DeviceScan::ExclusiveSum(tmp, b, len_t, rowptr_t, n + 1, s));
    if (nnz > 0) {
        // stable sort by (column, row): the rows of the transpose come out sorted by column
        b = tmp_bytes;
        GNN_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(tmp, b, keyA, keyB, entA, entB, (int)nnz, 0, key_bits, s));
        hipLaunchKernelGGL(k_transpose_out, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, nnz, keyB, entB, val, colidx_t, val_t);
    }
    GNN_HIP_TRY(hipGetLastError());
    GNN_HIP_TRY(hipStreamSynchronize(s));
    return GNN_OK;
}

int gnn_aes_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, int64_t *aes_sum, double *aes,
                   int *should_reorder, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) return GNN_EINVAL;
    if (nnz > 0 && (!rowptr || !colidx)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long host_total = 0;
    if (nnz > 0) {
        Arena mem;
        unsigned long long *total;
        mem.want(&total, 1);
        GNN_TRY(mem.commit());
        hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(kThreads), 0, s, (int *)total, (int64_t)2, 0);
        hipLaunchKernelGGL(k_aes_sum, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, n, nnz, rowptr, colidx, total);
        GNN_HIP_TRY(hipGetLastError());
        GNN_HIP_TRY(hipMemcpyAsync(&host_total, total, sizeof(host_total), hipMemcpyDeviceToHost, s));
        GNN_HIP_TRY(hipStreamSynchronize(s));
    }
    if (aes_sum) *aes_sum = (int64_t)host_total;
    if (aes) *aes = nnz > 0 ? (double)host_total / (double)nnz : 0.0;
    if (should_reorder) {
        // sqrt(AES) > floor(sqrt(n) / 100), compared in integers: sum > T^2 * nnz
        long long r = (long long)sqrt((double)n);
        while (r * r > (long long)n) --r;
        while ((r + 1) * (r + 1) <= (long long)n) ++r;
        const long long T = r / 100;
        *should_reorder = (long long)host_total > T * T * (long long)nnz ? 1 : 0;
    }
    return GNN_OK;
}

int gnn_gcn_norm_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float *ew, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) return GNN_EINVAL;
    if (nnz == 0) return GNN_OK;
    if (!rowptr || !colidx || !ew) return GNN_EINVAL;
    hipLaunchKernelGGL(k_gcn_norm, dim3(blocks_for(nnz)), dim3(kThreads), 0, (hipStream_t)stream, n, nnz, rowptr, colidx, ew);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

}  // extern "C"
