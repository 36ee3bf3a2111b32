// Pieces shared by the aggregation kernels: launch parameters, vector load/store, epilogue.
#ifndef GNN_AGG_COMMON_H
#define GNN_AGG_COMMON_H

#include <hip/hip_runtime.h>

#include "gnn_device.h"
#include "gnn_internal.h"

namespace gnn {

struct AggParams {
    WsHeader *hdr;
    const NgEntry *ng;
    const int *ngptr;
    const int *colidx;
    const float *ew;
    const float *evec;  // per-entry feature vectors [nnz, dim] multiplied into the neighbour rows elementwise, or null
    const float *X;
    float *out;
    float *part_rows;    // ordered flush: float[2 * tiles * dim] partial rows of spanning nodes; else null
    int *cnt;           // ordered flush: per-node arrival counters (zero on entry and on exit)
    const float *bias;  // epilogue: out = act(sum + bias); may be null
    const int *rowptr;  // mean aggregation: a finished row is divided by its length; null otherwise
    float self_scale;   // 1 + eps (GIN)
    int relu;
    int n;
    int dim;
    int ngs;
    int dwl_log2;
    int T;           // neighbor groups per block
    int iter_total;  // chunks of dwl*VEC floats per row
    int xcd_remap;
    int do_empty;    // 1: the main kernel writes the rows without entries; 0: the init kernel does
    int stream_out;  // 1: write output rows with streaming stores
    int plain_rows;  // 1: a finished row is stored as it is (no bias, activation or scaling) with streaming stores
    int full_rows;   // 1: one pass, every lane of a team in range: dim == chunks * dw * vector width
    int extra_blocks;  // blocks of the grid that serve the rows without entries (the first ones; the block-tile
                       // fused layer appends them)
    int64_t tile_blocks;  // blocks that serve tiles
    int64_t nnz;
    uint64_t rowptr_key;  // address of the caller's rowptr: the graph the stored partition must belong to
};

// Reduction over the neighbour rows (Sec. 3.1): sum (GCN, GIN; mean is a sum scaled when the row is
// written), or an elementwise max / min.
constexpr int kOpSum = 0, kOpMax = 1, kOpMin = 2;

template <int OP>
__device__ __forceinline__ float op_identity()
{
    if constexpr (OP == kOpMax) return -__builtin_inff();
    else if constexpr (OP == kOpMin) return __builtin_inff();
    else return 0.0f;
}

template <int OP>
__device__ __forceinline__ float op_combine(float a, float b)
{
    if constexpr (OP == kOpMax) return fmaxf(a, b);
    else if constexpr (OP == kOpMin) return fminf(a, b);
    else return a + b;
}

template <int VEC>
__device__ __forceinline__ void load_vec(float (&r)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else if constexpr (VEC == 2) {
        const float2 v = *reinterpret_cast<const float2 *>(p);
        r[0] = v.x; r[1] = v.y;
    } else {
        r[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&r)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(r[0], r[1], r[2], r[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(r[0], r[1]);
    } else {
        *p = r[0];
    }
}

// Partial rows of the ordered flush travel between blocks that may run on different XCDs, whose L2
// caches are not coherent with each other for ordinary accesses.  They are therefore written and
// read with device-scope relaxed atomic accesses (write-through stores, cache-missing loads): no
// cache-wide write-back or invalidate is needed, only the order store -> counter -> load.
template <int VEC>
__device__ __forceinline__ void store_vec_coherent(float *p, const float (&r)[VEC])
{
#pragma unroll
    for (int j = 0; j < VEC; ++j) __hip_atomic_store(p + j, r[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int VEC>
__device__ __forceinline__ void load_vec_coherent(float (&r)[VEC], const float *p)
{
#pragma unroll
    for (int j = 0; j < VEC; ++j) r[j] = __hip_atomic_load(p + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#ifndef GNN_NT_STORE
#define GNN_NT_STORE 1
#endif
#ifndef GNN_NT_INDEX
#define GNN_NT_INDEX 1
#endif

// Output rows are written once and not read again by the kernel: a streaming (non-temporal) store
// keeps them from displacing neighbour rows in the caches.
template <int VEC>
__device__ __forceinline__ void store_vec_stream(float *p, const float (&r)[VEC])
{
#if GNN_NT_STORE
    typedef float v4 __attribute__((ext_vector_type(4)));
    typedef float v2 __attribute__((ext_vector_type(2)));
    if constexpr (VEC == 4) {
        v4 v = {r[0], r[1], r[2], r[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<v4 *>(p));
    } else if constexpr (VEC == 2) {
        v2 v = {r[0], r[1]};
        __builtin_nontemporal_store(v, reinterpret_cast<v2 *>(p));
    } else {
        __builtin_nontemporal_store(r[0], p);
    }
#else
    store_vec<VEC>(p, r);
#endif
}

// A row that is read exactly once (a node's own row, the rows without entries): streaming load.
template <int VEC>
__device__ __forceinline__ void load_vec_stream(float (&r)[VEC], const float *p)
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    typedef float v2 __attribute__((ext_vector_type(2)));
    if constexpr (VEC == 4) {
        const v4 t = __builtin_nontemporal_load(reinterpret_cast<const v4 *>(p));
        r[0] = t[0]; r[1] = t[1]; r[2] = t[2]; r[3] = t[3];
    } else if constexpr (VEC == 2) {
        const v2 t = __builtin_nontemporal_load(reinterpret_cast<const v2 *>(p));
        r[0] = t[0]; r[1] = t[1];
    } else {
        r[0] = __builtin_nontemporal_load(p);
    }
}

// Column indices, edge weights and group tuples are read exactly once.
template <typename T>
__device__ __forceinline__ T load_stream(const T *p)
{
#if GNN_NT_INDEX
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// The header words a kernel checks before it trusts the partition, read in one go.
struct HeaderVals {
    uint32_t magic;
    int32_t n, ngs, status;
    int64_t nnz, num_ng;
    uint64_t rowptr_addr;
};

__device__ __forceinline__ HeaderVals load_header(const WsHeader *hdr)
{
    HeaderVals h;
    h.magic = hdr->magic;
    h.n = hdr->n;
    h.ngs = hdr->ngs;
    h.status = hdr->status;
    h.nnz = hdr->nnz;
    h.num_ng = hdr->num_ng;
    h.rowptr_addr = hdr->rowptr_addr;
    return h;
}

__device__ __forceinline__ bool header_vals_ok(const HeaderVals &h, const AggParams &p)
{
    // (n, nnz, ngs) alone would accept the partition of another graph of the same size -- a renumbered
    // graph keeps both -- so the partition is also tied to the rowptr array it was built from
    return (h.magic == kMagic) & (h.status == GNN_OK) & (h.ngs == p.ngs) & (h.n == p.n) & (h.nnz == p.nnz) &
           (h.rowptr_addr == p.rowptr_key);
}

__device__ __forceinline__ bool header_ok(const WsHeader *hdr, const AggParams &p)
{
    return header_vals_ok(load_header(hdr), p);
}

// The workspace does not hold the partition the launch was prepared for: record why nothing was
// computed (one thread).
__device__ __forceinline__ void note_stale(WsHeader *hdr, const AggParams &p)
{
    if (hdr->magic != kMagic) {
        hdr->magic = kMagic;
        hdr->n = p.n;
        hdr->nnz = p.nnz;
        hdr->ngs = 0;
        hdr->num_ng = 0;
        hdr->status = GNN_ESTALE;
    } else if (hdr->status == GNN_OK) {
        hdr->status = GNN_ESTALE;
    }
}

// 1 / (row length) for the mean aggregation, 1 otherwise.
__device__ __forceinline__ float row_scale(const AggParams &p, int node)
{
    if (!p.rowptr) return 1.0f;
    return 1.0f / (float)(p.rowptr[node + 1] - p.rowptr[node]);
}

__device__ __forceinline__ float epilogue(float v, const float *bias, int d, int relu)
{
    if (bias) v += bias[d];
    if (relu) v = fmaxf(v, 0.0f);
    return v;
}

// Rows without any entry: out = act((1+eps) x + b) (GIN) or act(b).  The calling wave scans chunks
// of 64 nodes (first_chunk, first_chunk + chunk_stride, ...), lists the empty ones in `mylist`
// (64 ints of LDS private to the wave) and lets its teams write them side by side, four rows per
// team in flight.
template <int VEC, bool SELF>
__device__ __forceinline__ void write_empty_rows(const AggParams &p, int64_t first_chunk, int64_t chunk_stride,
                                                 int *mylist)
{
    const int lane = threadIdx.x & 63;
    const int dwl = 1 << p.dwl_log2, G = 64 >> p.dwl_log2;
    const int tlane = lane & (dwl - 1), team_in_wave = lane >> p.dwl_log2;
    const int dim = p.dim;
    const int64_t nchunks = ((int64_t)p.n + 63) / 64;
    for (int64_t c = first_chunk; c < nchunks; c += chunk_stride) {
        const int64_t v = c * 64 + lane;
        const bool empty = v < p.n && p.ngptr[v] == p.ngptr[v + 1];
        const unsigned long long m = __ballot(empty);
        if (m == 0ull) continue;
        const int cnt = __popcll(m);
        if (empty) mylist[__popcll(m & ((1ull << lane) - 1ull))] = lane;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int k0 = team_in_wave; k0 < cnt; k0 += 4 * G) {
            int64_t node[4];
            bool ok[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int k = k0 + q * G;
                ok[q] = k < cnt;
                node[q] = c * 64 + (ok[q] ? mylist[k] : 0);
            }
            for (int cc = 0; cc < p.iter_total; ++cc) {
                const int d = (cc * dwl + tlane) * VEC;
                if (d >= dim) break;
                float r[4][VEC];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) r[q][j] = 0.0f;
                    // (read once: a streaming load keeps these rows from displacing the hubs' rows in L2)
                    if (SELF && ok[q]) load_vec_stream<VEC>(r[q], p.X + (size_t)node[q] * dim + d);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (ok[q]) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j)
                            r[q][j] = epilogue(SELF ? p.self_scale * r[q][j] : 0.0f, p.bias, d + j, p.relu);
                        if (p.stream_out) store_vec_stream<VEC>(p.out + (size_t)node[q] * dim + d, r[q]);
                        else store_vec<VEC>(p.out + (size_t)node[q] * dim + d, r[q]);
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace gnn
#endif
