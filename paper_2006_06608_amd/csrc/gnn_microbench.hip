// Two measuring kernels for the memory system, so that a benchmark can state what this machine
// delivers for the aggregation's access patterns next to the published peak: a read-only stream and a
// bare gather of feature rows (the aggregation kernel's loads without tuples, reduction or stores).
#include <hip/hip_runtime.h>

#include "gnn_bench.h"
#include "gnn_internal.h"

namespace gnn {

__global__ __launch_bounds__(256) void k_bench_stream_read(const float4 *__restrict__ a, size_t n4, float *sink)
{
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {  // four independent loads in flight per lane
        const float4 v0 = a[i], v1 = a[i + stride], v2 = a[i + 2 * stride], v3 = a[i + 3 * stride];
        acc.x += v0.x + v1.x + v2.x + v3.x;
        acc.y += v0.y + v1.y + v2.y + v3.y;
        acc.z += v0.z + v1.z + v2.z + v3.z;
        acc.w += v0.w + v1.w + v2.w + v3.w;
    }
    for (; i < n4; i += stride) {
        const float4 v = a[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    // never true for finite data, but keeps the loads alive
    if (acc.x + acc.y + acc.z + acc.w == 1.2345678e38f) sink[0] = acc.x;
}

// A team of 2^team_log2 lanes reads rows idx[k] of dim = 4 * 2^team_log2 * chunks floats, eight rows in
// flight per chunk, as the aggregation kernel's teams do.
__global__ __launch_bounds__(256) void k_bench_gather_rows(const float *__restrict__ X, int dim, int team_log2, int chunks,
                                                           const int *__restrict__ idx, int64_t nidx, float *sink)
{
    const int tlane = threadIdx.x & ((1 << team_log2) - 1);
    const int64_t team = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> team_log2;
    const int64_t nteams = ((int64_t)gridDim.x * blockDim.x) >> team_log2;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t base = team * 8; base + 8 <= nidx; base += nteams * 8) {
        int c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = idx[base + u];
        for (int ch = 0; ch < chunks; ++ch) {
            const int d = ((ch << team_log2) + tlane) * 4;
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4 *>(X + (size_t)(unsigned)c[u] * (unsigned)dim + d);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w;
            }
        }
    }
    if (acc.x + acc.y + acc.z + acc.w == 1.2345678e38f) sink[0] = acc.x;
}

}  // namespace gnn

using namespace gnn;

extern "C" {

int gnn_bench_stream_read(const void *src, size_t bytes, float *sink, void *stream)
{
    if (!src || !sink || ((uintptr_t)src & 15) != 0) return GNN_EINVAL;
    hipLaunchKernelGGL(k_bench_stream_read, dim3(8192), dim3(256), 0, (hipStream_t)stream, (const float4 *)src, bytes / 16, sink);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

int gnn_bench_gather_rows(int32_t n, int32_t dim, const float *X, const int32_t *idx, int64_t nidx, float *sink, void *stream)
{
    if (n <= 0 || nidx < 0 || !X || !sink || (nidx > 0 && !idx) || ((uintptr_t)X & 15) != 0) return GNN_EINVAL;
    // dim = 4 floats x team (a power of two up to 64 lanes) x chunks (1..4), the widest team first
    int team_log2 = -1, chunks = 0;
    for (int t = 6; t >= 0 && team_log2 < 0; --t)
        for (int c = 1; c <= 4; ++c)
            if (dim == 4 * (1 << t) * c) {
                team_log2 = t;
                chunks = c;
                break;
            }
    if (team_log2 < 0) return GNN_EINVAL;
    hipLaunchKernelGGL(k_bench_gather_rows, dim3(16384), dim3(256), 0, (hipStream_t)stream, X, dim, team_log2, chunks, idx, nidx,
                       sink);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

}  // extern "C"
