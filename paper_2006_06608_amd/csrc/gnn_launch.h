// Host-side functions that the translation units of the library call in each other (HIP types,
// hence separate from gnn_internal.h, which the plain C++ host file includes too).
#ifndef GNN_LAUNCH_H
#define GNN_LAUNCH_H

#include <hip/hip_runtime.h>

#include "gnn_agg_common.h"

namespace gnn {

// gnn_partition.hip: neighbor partitioning of rowptr into the workspace (Sec. 4.1).
int partition_build_impl(int32_t n, int64_t nnz, const int32_t *rowptr, int32_t ngs, void *workspace,
                         size_t workspace_bytes, hipStream_t s);

// gnn_aggregate.hip: shared implementation of gnn_aggregate_gcn / gnn_aggregate_gin and of the
// aggregation step of the layer entry points.  self: add self_scale * X[i] (GIN).  bias/relu: fused
// epilogue.  ws_reserved: bytes at the front of the workspace that the caller uses itself (0: only
// the partition); the partial rows of the ordered flush are placed behind them.  ev_start/ev_stop
// (may be null) are recorded around the main kernel.  fuse (may be null): see FuseSpec.
// op: kOpSum / kOpMax / kOpMin; mean: divide every finished row by its length (op must be kOpSum).
// Anything but the plain sum takes no weights, no self term, and needs the ordered flush.
// evec (may be null): per-entry feature vectors [nnz, dim], multiplied into the neighbour rows elementwise.
int aggregate_reduce_impl(int op, bool mean, bool self, float self_scale, int32_t n, int64_t nnz, const int32_t *rowptr,
                          const int32_t *colidx, const float *ew, const float *X, float *out, int32_t dim, int32_t ngs,
                          int32_t dw, int32_t wpb, uint32_t flags, const float *bias, int relu, void *workspace,
                          size_t workspace_bytes, size_t ws_reserved, hipStream_t s, hipEvent_t ev_start,
                          hipEvent_t ev_stop, FuseSpec *fuse, const float *evec = nullptr);

inline int aggregate_impl(bool self, float self_scale, int32_t n, int64_t nnz, const int32_t *rowptr,
                          const int32_t *colidx, const float *ew, const float *X, float *out, int32_t dim, int32_t ngs,
                          int32_t dw, int32_t wpb, uint32_t flags, const float *bias, int relu, void *workspace,
                          size_t workspace_bytes, size_t ws_reserved, hipStream_t s, hipEvent_t ev_start,
                          hipEvent_t ev_stop, FuseSpec *fuse)
{
    return aggregate_reduce_impl(kOpSum, false, self, self_scale, n, nnz, rowptr, colidx, ew, X, out, dim, ngs, dw, wpb,
                                 flags, bias, relu, workspace, workspace_bytes, ws_reserved, s, ev_start, ev_stop, fuse);
}
void launch_agg_init(const AggParams &p, bool self, hipStream_t s);
void launch_agg_epilogue_spanning(const AggParams &p, hipStream_t s);

// gnn_gin_fused.hip: GIN aggregation with the Update fused in, on the general kernel with the ordered
// flush; p.part_rows must have room for rows of max(p.dim, M) floats.  Returns GNN_OK when the fused
// kernel was launched, 1 when the shape does not qualify (nothing launched), < 0 on error.
// waves_used (may be null) receives the waves per block of the kernel that was launched.
int try_gin_layer_fused(AggParams &p, int vec, int wpb, const float *W, const float *b, float *out, int M, int relu,
                        int64_t tiles_upper, hipStream_t s, int *waves_used);
// true if the wave-tile form of the fused layer covers the shape; the caller then sets p.T = 16 and sizes the
// partial rows for tiles of 16 groups before it calls try_gin_layer_fused
bool gin_layer_fused_wave_tiles(const AggParams &p, int vec, int M);

// gnn_update.hip: out[n,M] = act(A[n,K] W[K,M] + b) on the MFMA units.
int update_gemm_impl(int32_t n, int32_t K, int32_t M, const float *A, const float *W, const float *b, int relu,
                     float *out, hipStream_t s);

}  // namespace gnn
#endif
