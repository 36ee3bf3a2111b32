// Neighbor partitioning on the device (Sec. 4.1): per-node group counts, their prefix sum, and
// the neighbor-partitioning graph store (one NgEntry per group).  Also CSR validation and the
// exports used by tests.
#include <hip/hip_runtime.h>

#include <vector>

#include "gnn_device.h"
#include "gnn_launch.h"

namespace gnn {

constexpr int kScanThreads = 256;
constexpr int kScanPerThread = kScanTile / kScanThreads;  // 8

__device__ __forceinline__ int groups_of(int deg, int ngs) { return (deg + ngs - 1) / ngs; }

// Block-wide inclusive scan of one int per thread (256 threads), returns the inclusive value;
// total receives the block sum.
__device__ __forceinline__ int block_scan_incl(int v, int *s_wave, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    if (lane == 63) s_wave[wave] = x;
    __syncthreads();
    int base = 0;
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        const int s = s_wave[w];
        if (w < wave) base += s;
        tot += s;
    }
    total = tot;
    __syncthreads();
    return x + base;
}

__global__ void k_reset_header(WsHeader *hdr)
{
    // a kernel rather than a memset node, so that callers may capture the call in a HIP graph
    hdr->magic = 0;
    hdr->status = GNN_OK;
    hdr->num_ng = 0;
}

// Pass 1: group count of every tile of kScanTile nodes; flags a decreasing rowptr.
__global__ __launch_bounds__(kScanThreads) void k_count_tiles(int n, const int *__restrict__ rowptr, int ngs,
                                                              int *__restrict__ tile_sum, WsHeader *hdr)
{
    __shared__ int s_wave[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    int cnt = 0;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        const int64_t v = base + (int64_t)k * kScanThreads + threadIdx.x;
        if (v < n) {
            const int d = rowptr[v + 1] - rowptr[v];
            if (d < 0) bad = true;
            else cnt += groups_of(d, ngs);
        }
    }
    if (bad) hdr->status = GNN_ECSR;
    int total;
    block_scan_incl(cnt, s_wave, total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// Pass 2 (one block): exclusive scan of the tile sums in place; writes the header.
__global__ __launch_bounds__(kScanThreads) void k_scan_tiles(int64_t tiles, int *__restrict__ tile_sum, WsHeader *hdr,
                                                             int n, int64_t nnz, int ngs, int64_t capacity,
                                                             const int *__restrict__ rowptr)
{
    __shared__ int s_wave[kScanThreads / 64];
    int64_t carry = 0;
    for (int64_t b0 = 0; b0 < tiles; b0 += kScanThreads) {
        const int64_t i = b0 + threadIdx.x;
        const int v = i < tiles ? tile_sum[i] : 0;
        int total;
        const int incl = block_scan_incl(v, s_wave, total);
        if (i < tiles) tile_sum[i] = (int)(carry + incl - v);
        carry += total;
    }
    if (threadIdx.x == 0) {
        tile_sum[tiles] = (int)carry;
        int status = hdr->status;
        if (n > 0 && (rowptr[0] != 0 || (int64_t)rowptr[n] != nnz)) status = GNN_ECSR;
        if (n == 0 && nnz != 0) status = GNN_ECSR;
        if (carry > capacity) status = GNN_ECSR;  // cannot happen for a consistent (rowptr, nnz)
        hdr->magic = kMagic;
        hdr->n = n;
        hdr->nnz = nnz;
        hdr->ngs = ngs;
        hdr->status = status;
        hdr->num_ng = status == GNN_OK ? carry : 0;
        hdr->ng_capacity = capacity;
        hdr->rowptr_addr = (uint64_t)rowptr;
    }
}

// Pass 3: ngptr[v] = id of the first neighbor group of node v; the arrival counters of the ordered
// flush start at zero.
__global__ __launch_bounds__(kScanThreads) void k_fill_ngptr(int n, const int *__restrict__ rowptr, int ngs,
                                                             const int *__restrict__ tile_off, int *__restrict__ ngptr,
                                                             int *__restrict__ cnt, const WsHeader *hdr)
{
    __shared__ int s_wave[kScanThreads / 64];
    if (hdr->status != GNN_OK) return;
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    // thread t owns kScanPerThread consecutive nodes, so that one scan over per-thread sums suffices
    const int64_t v0 = base + (int64_t)threadIdx.x * kScanPerThread;
    int c[kScanPerThread];
    int mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        const int64_t v = v0 + k;
        c[k] = v < n ? groups_of(rowptr[v + 1] - rowptr[v], ngs) : 0;
        mine += c[k];
    }
    int total;
    const int incl = block_scan_incl(mine, s_wave, total);
    int run = tile_off[blockIdx.x] + incl - mine;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        const int64_t v = v0 + k;
        if (v < n) {
            ngptr[v] = run;
            cnt[v] = 0;
        }
        run += c[k];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) ngptr[n] = tile_off[gridDim.x];
}

// Pass 4: one thread per neighbor group: find its node by bisection on ngptr, write the tuple.
__global__ __launch_bounds__(256) void k_fill_groups(int n, const int *__restrict__ rowptr, int ngs,
                                                     const int *__restrict__ ngptr, NgEntry *__restrict__ ng,
                                                     const WsHeader *hdr)
{
    if (hdr->status != GNN_OK) return;
    const int64_t num_ng = hdr->num_ng;
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= num_ng) return;
    // largest v with ngptr[v] <= g (nodes without groups share their successor's value and are skipped)
    int lo = 0, hi = n;  // invariant: ngptr[lo] <= g < ngptr[hi]
    while (hi - lo > 1) {
        const int mid = lo + ((hi - lo) >> 1);
        if (ngptr[mid] <= (int)g) lo = mid;
        else hi = mid;
    }
    const int v = lo;
    const int j = (int)g - ngptr[v];
    const int r0 = rowptr[v], r1 = rowptr[v + 1];
    const int start = r0 + j * ngs;
    const int end = min(start + ngs, r1);
    NgEntry e;
    e.node = v;
    e.start = start;
    e.end = end;
    e.flags = (start == r0 ? 1 : 0) | (end == r1 ? 2 : 0);
    ng[g] = e;
}

__global__ __launch_bounds__(256) void k_validate_csr(int n, int64_t nnz, const int *__restrict__ rowptr,
                                                      const int *__restrict__ colidx, int *bad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool b = false;
    if (i == 0 && n >= 0) {
        if (rowptr[0] != 0 || (int64_t)rowptr[n] != nnz) b = true;
    }
    for (int64_t v = i; v < n; v += stride)
        if (rowptr[v + 1] < rowptr[v]) b = true;
    // only walk colidx when rowptr[n] agrees with nnz (otherwise the length is unknown)
    if ((int64_t)rowptr[n] == nnz)
        for (int64_t e = i; e < nnz; e += stride) {
            const int c = colidx[e];
            if (c < 0 || c >= n) b = true;
        }
    if (b) *bad = 1;
}

// Algorithm 1 as the aggregation kernel evaluates it, written out per neighbor group.
__global__ void k_export_layout(const WsHeader *hdr, const NgEntry *__restrict__ ng, int groups_per_block,
                                int dwl_log2, int *__restrict__ slot_out, unsigned char *__restrict__ leader_out)
{
    extern __shared__ int s_lay[];
    const int64_t num_ng = hdr->num_ng;
    const int64_t g0 = (int64_t)blockIdx.x * groups_per_block;
    if (g0 >= num_ng) return;
    const BlockLayout lay = block_layout(ng, g0, num_ng, dwl_log2, s_lay);
    __syncthreads();
    const int slot = block_layout_slot(lay, dwl_log2, s_lay);
    const int tlane = threadIdx.x & ((1 << dwl_log2) - 1);
    if (lay.valid && tlane == 0) {
        slot_out[lay.g] = slot;
        leader_out[lay.g] = lay.leader ? 1 : 0;
    }
}

static int check_ws(const void *workspace, size_t bytes, size_t need)
{
    if (!workspace) return GNN_EWORKSPACE;
    if (((uintptr_t)workspace) % kAlign != 0) return GNN_EWORKSPACE;
    if (bytes < need) return GNN_EWORKSPACE;
    return GNN_OK;
}

int partition_build_impl(int32_t n, int64_t nnz, const int32_t *rowptr, int32_t ngs, void *workspace,
                         size_t workspace_bytes, hipStream_t s)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31) || ngs < 1 || !rowptr) return GNN_EINVAL;
    const WsLayout L = ws_layout(n, nnz, 0, ngs);
    const int rc = check_ws(workspace, workspace_bytes, L.total);
    if (rc != GNN_OK) return rc;
    char *ws = (char *)workspace;
    WsHeader *hdr = (WsHeader *)(ws + L.header);
    int *ngptr = (int *)(ws + L.ngptr);
    int *cnt = (int *)(ws + L.cnt);
    int *scan = (int *)(ws + L.scan);
    NgEntry *ng = (NgEntry *)(ws + L.ng);
    // header starts from a clean status; the scan kernel fills the rest
    hipLaunchKernelGGL(k_reset_header, dim3(1), dim3(1), 0, s, hdr);
    const int64_t tiles = L.scan_blocks;
    if (tiles > 0) {
        hipLaunchKernelGGL(k_count_tiles, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, n, rowptr, ngs, scan, hdr);
    }
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(kScanThreads), 0, s, tiles, scan, hdr, n, nnz, ngs, L.ng_capacity,
                       rowptr);
    if (tiles > 0) {
        hipLaunchKernelGGL(k_fill_ngptr, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, n, rowptr, ngs, scan, ngptr,
                           cnt, hdr);
        const int64_t blocks = (L.ng_capacity + 255) / 256;
        if (blocks > 0)
            hipLaunchKernelGGL(k_fill_groups, dim3((unsigned)blocks), dim3(256), 0, s, n, rowptr, ngs, ngptr, ng, hdr);
    }
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" {

size_t gnn_workspace_bytes(int32_t n, int64_t nnz, int32_t max_dim, int32_t ngs)
{
    if (n < 0 || nnz < 0 || max_dim < 0 || ngs < 0) return 0;
    const WsLayout L = ws_layout(n, nnz, max_dim, ngs);
    return L.total + part_rows_bytes(L.ng_capacity, kPartMinTile, max_dim);
}

int gnn_partition_build(int32_t n, int64_t nnz, const int32_t *rowptr, int32_t ngs, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    return partition_build_impl(n, nnz, rowptr, ngs, workspace, workspace_bytes, (hipStream_t)stream);
}

int gnn_workspace_status(const void *workspace, void *stream, int64_t *num_ng, int32_t *ngs)
{
    if (!workspace) return GNN_EWORKSPACE;
    WsHeader h;
    GNN_HIP_TRY(hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, (hipStream_t)stream));
    GNN_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    if (h.magic != kMagic) return GNN_ESTALE;
    if (num_ng) *num_ng = h.num_ng;
    if (ngs) *ngs = h.ngs;
    return h.status;
}

int gnn_partition_export(const void *workspace, void *stream, int64_t capacity, int32_t *ng_node, int32_t *ng_start,
                         int32_t *ng_end)
{
    if (!workspace || capacity < 0) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    WsHeader h;
    GNN_HIP_TRY(hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, s));
    GNN_HIP_TRY(hipStreamSynchronize(s));
    if (h.magic != kMagic) return GNN_ESTALE;
    if (h.status != GNN_OK) return h.status;
    if (h.num_ng > capacity) return GNN_ELIMIT;
    if (h.num_ng == 0) return GNN_OK;
    if (!ng_node || !ng_start || !ng_end) return GNN_EINVAL;
    const WsLayout L = ws_layout(h.n, h.nnz, 0, h.ngs);
    std::vector<NgEntry> host((size_t)h.num_ng);
    GNN_HIP_TRY(hipMemcpyAsync(host.data(), (const char *)workspace + L.ng, sizeof(NgEntry) * (size_t)h.num_ng,
                               hipMemcpyDeviceToHost, s));
    GNN_HIP_TRY(hipStreamSynchronize(s));
    for (int64_t g = 0; g < h.num_ng; ++g) {
        ng_node[g] = host[g].node;
        ng_start[g] = host[g].start;
        ng_end[g] = host[g].end;
    }
    return GNN_OK;
}

int gnn_block_layout_export(const void *workspace, void *stream, int32_t dim, int32_t dw, int32_t waves_per_block,
                            int64_t capacity, int32_t *slot, uint8_t *leader, int32_t *groups_per_block)
{
    if (!workspace || dim <= 0 || capacity < 0) return GNN_EINVAL;
    if (dw < 1 || dw > 64 || (dw & (dw - 1)) != 0) return GNN_EINVAL;
    if (waves_per_block < 1 || waves_per_block > kMaxWavesPerBlock) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    WsHeader h;
    GNN_HIP_TRY(hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, s));
    GNN_HIP_TRY(hipStreamSynchronize(s));
    if (h.magic != kMagic) return GNN_ESTALE;
    if (h.status != GNN_OK) return h.status;
    int dwl_log2 = 0;
    while ((1 << dwl_log2) < dw) ++dwl_log2;
    const int T = waves_per_block * (64 >> dwl_log2);
    if (groups_per_block) *groups_per_block = T;
    if (h.num_ng > capacity) return GNN_ELIMIT;
    if (h.num_ng == 0) return GNN_OK;
    if (!slot || !leader) return GNN_EINVAL;
    const WsLayout L = ws_layout(h.n, h.nnz, 0, h.ngs);
    int *d_slot = nullptr;
    unsigned char *d_leader = nullptr;
    // test/diagnostic path: temporary device buffers are acceptable here (never on the hot path)
    GNN_HIP_TRY(hipMalloc(&d_slot, sizeof(int) * (size_t)h.num_ng));
    if (hipMalloc(&d_leader, (size_t)h.num_ng) != hipSuccess) {
        (void)hipFree(d_slot);
        return GNN_EHIP;
    }
    const int64_t blocks = (h.num_ng + T - 1) / T;
    hipLaunchKernelGGL(k_export_layout, dim3((unsigned)blocks), dim3(waves_per_block * 64),
                       sizeof(int) * (size_t)(waves_per_block + 1), s, (const WsHeader *)workspace,
                       (const NgEntry *)((const char *)workspace + L.ng), T, dwl_log2, d_slot, d_leader);
    hipError_t e1 = hipMemcpyAsync(slot, d_slot, sizeof(int) * (size_t)h.num_ng, hipMemcpyDeviceToHost, s);
    hipError_t e2 = hipMemcpyAsync(leader, d_leader, (size_t)h.num_ng, hipMemcpyDeviceToHost, s);
    hipError_t e3 = hipStreamSynchronize(s);
    (void)hipFree(d_slot);
    (void)hipFree(d_leader);
    if (e1 != hipSuccess) GNN_HIP_TRY(e1);
    if (e2 != hipSuccess) GNN_HIP_TRY(e2);
    if (e3 != hipSuccess) GNN_HIP_TRY(e3);
    return GNN_OK;
}

int gnn_validate_csr_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, void *stream)
{
    if (n < 0 || nnz < 0 || nnz >= ((int64_t)1 << 31) || !rowptr || (nnz > 0 && !colidx)) return GNN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int *d_bad = nullptr;
    GNN_HIP_TRY(hipMalloc(&d_bad, sizeof(int)));
    hipError_t e = hipMemsetAsync(d_bad, 0, sizeof(int), s);
    int bad = 0;
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_validate_csr, dim3(1024), dim3(256), 0, s, n, nnz, rowptr, colidx, d_bad);
        e = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, s);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(d_bad);
    GNN_HIP_TRY(e);
    return bad ? GNN_ECSR : GNN_OK;
}

}  // extern "C"
