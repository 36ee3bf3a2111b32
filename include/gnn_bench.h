/*
 * gnn_bench.h -- measuring aids of the MI355X GNN aggregation library (same shared library as gnn.h).
 *
 * Nothing here is part of the computation: these entry points exist so that a benchmark can time the
 * aggregation kernel inside a running layer without a profiler and can quote, beside the published
 * peak, what the memory system of the machine at hand delivers for a plain stream and for a bare row
 * gather.  Conventions (status codes, HOST / DEVICE pointers, streams) are those of gnn.h.
 */
#ifndef GNN_MI355X_BENCH_H
#define GNN_MI355X_BENCH_H

#include "gnn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* gnn_layer_forward with two timing taps: ev_agg_start / ev_agg_stop (hipEvent_t, either may be
 * NULL) are recorded on `stream` immediately before and after the main aggregation kernel of
 * the layer, so that a benchmark can time that kernel inside a running model without a
 * profiler.  Everything else is identical to gnn_layer_forward. */
int gnn_layer_forward_timed(int kind, int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                            const float *ew, float eps, const float *X, int32_t in_dim, const float *W,
                            const float *b, int32_t out_dim, int relu, float *out, int32_t ngs, int32_t dw,
                            int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                            void *stream, void *ev_agg_start, void *ev_agg_stop);

/* What the memory system delivers.  Both only enqueue a kernel; the caller times it.
 * sink: DEVICE float[1], never written for finite data.
 * gnn_bench_stream_read: reads `bytes` (16-byte aligned src) once, sequentially.
 * gnn_bench_gather_rows: teams of lanes read the rows idx[0..nidx) of X[n, dim] with 16-byte
 * loads, eight rows in flight per team (the aggregation kernel's loads without its tuples, reduction
 * and stores); dim = 4 x (a power of two up to 64) x (1..4), e.g. 16, 64, 96, 256; 0 <= idx[k] < n is the
 * caller's duty; nidx is rounded down to a multiple of 8. */
int gnn_bench_stream_read(const void *src, size_t bytes, float *sink, void *stream);
int gnn_bench_gather_rows(int32_t n, int32_t dim, const float *X, const int32_t *idx, int64_t nidx, float *sink,
                          void *stream);

/* Which aggregation kernel the calling thread's last gnn_aggregate_* / gnn_layer_forward / gnn_model_forward
 * call enqueued, with its template arguments and launch shape, as text in buf (HOST, cap bytes), e.g.
 * "k_aggregate<4,1,8,4,false,true,0> groups/block=16 ngs=32 waves/block=4 flush=ordered tiles=xcd-runs".  A
 * benchmark uses it to tie counter readings taken with a profiler to the build that is being timed.
 * Errors: GNN_EINVAL (NULL), GNN_ELIMIT (cap too small). */
int gnn_bench_last_aggregation(char *buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* GNN_MI355X_BENCH_H */
