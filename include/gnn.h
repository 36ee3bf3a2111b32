/*
 * gnn.h -- C ABI of the MI355X (gfx950) GNN aggregation library.
 *
 * The library computes the Aggregation phase of a GNN layer (GNNAdvisor, arXiv 2006.06608):
 * a CSR sparse x dense product over fp32 node embeddings, with the paper's 2D workload
 * management (neighbor groups x dimension workers, Sec. 4), block-level scratch-memory
 * accumulation with leader flush (Sec. 5.2, Algorithm 1), community-aware renumbering
 * (Sec. 5.1) and a parameter model (Sec. 6), plus the dense Update so that a whole layer
 * can be run.
 *
 * Conventions
 *   - Every function returns GNN_OK (0) or a negative error code; none throws, aborts or
 *     prints.  gnn_strerror() names a code; gnn_last_hip_error() gives the HIP status
 *     behind the calling thread's last GNN_EHIP.
 *   - "HOST" / "DEVICE" on a pointer says where the memory must live.  The caller owns
 *     every buffer and the library keeps no state between calls.  The compute entry points
 *     allocate nothing; only the diagnostic calls that copy results to the host
 *     (gnn_block_layout_export, gnn_validate_csr_device) and the one-time graph preparation on
 *     the device (gnn_reorder_device, gnn_apply_perm_csr_device, gnn_csr_transpose_device, gnn_aes_device) use
 *     temporary device buffers.
 *   - Matrices are row-major fp32; CSR indices are int32 (nnz < 2^31); n * dim is
 *     addressed in 64 bits.  In and out buffers must not alias.
 *   - DEVICE entry points only enqueue work on `stream` (a hipStream_t, NULL = the null
 *     stream) and return without synchronising, unless stated otherwise.  Errors that can
 *     be seen at enqueue time are returned; a malformed device-side CSR (rowptr[n] != nnz,
 *     decreasing rowptr) is caught by the partition kernels, recorded in the workspace and
 *     reported by gnn_workspace_status(); column indices outside [0, n) are only caught by
 *     gnn_validate_csr_device(), which callers of untrusted graphs must run first.
 */
#ifndef GNN_MI355X_H
#define GNN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---------------------------------------------------------------- */
#define GNN_OK 0
#define GNN_EINVAL (-1)     /* NULL or out-of-range argument                              */
#define GNN_ECSR (-2)       /* malformed CSR                                              */
#define GNN_EWORKSPACE (-3) /* workspace missing, misaligned (256 B) or too small         */
#define GNN_EHIP (-4)       /* a HIP runtime call failed                                  */
#define GNN_ELIMIT (-5)     /* parameters exceed a documented limit (LDS budget, sizes)   */
#define GNN_ESTALE (-6)     /* GNN_FLAG_REUSE_PARTITION but the workspace holds no partition for (rowptr, n, nnz, ngs) */

/* ---- layer kinds (Sec. 3.1) ------------------------------------------------------ */
#define GNN_GCN 0 /* Update (GEMM), then Aggregation (Eq. 2), then bias/activation */
#define GNN_GIN 1 /* Aggregation (Eq. 3), then Update (GEMM + bias), then activation */

/* ---- flags of the DEVICE entry points -------------------------------------------- */
#define GNN_FLAG_REUSE_PARTITION 1u /* workspace already holds the neighbor partition for this
                                       (rowptr, ngs), built by gnn_partition_build or by an earlier
                                       call without this flag: the one-time preparation of Sec. 4.1.
                                       The partition is tied to the ADDRESS of the rowptr array it was
                                       built from (and to n, nnz, ngs): a call with another rowptr array
                                       computes nothing and gnn_workspace_status reports GNN_ESTALE.
                                       Changing the contents of that array in place is the caller's
                                       responsibility (build the partition again) */
#define GNN_FLAG_NO_BLOCK_OPT 2u    /* ablation (Sec. 7.4 "block-level optimization"): no scratch-memory
                                       slots, no leaders; every neighbor group adds to global memory */
#define GNN_FLAG_XCD_RUNS 4u        /* block-to-tile order that keeps runs of 32 consecutive tiles on one
                                       XCD (one L2) instead of dealing consecutive tiles round-robin over
                                       the eight XCDs: fewer bytes fetched beyond L2 on graphs whose ids
                                       follow communities, 1-3 % less run time.  The library uses this
                                       order by itself from ngs = 16 on; the flag asks for it with smaller
                                       groups too (measured slower there) */
#define GNN_FLAG_NO_PIPELINE 8u     /* accepted and ignored (kept for callers of an earlier version, which had */
#define GNN_FLAG_PIPELINE 16u       /* a second, persistent kernel that these two flags forbade / forced)      */
#define GNN_FLAG_DETERMINISTIC 32u  /* require the ordered flush (bitwise identical results from run to run
                                       for fixed ngs, dw, waves): no float atomics.  The waves of a block add
                                       to a shared slot in wave order; a block leaves the partial rows of nodes
                                       that span blocks in scratch memory behind the caller's use of the
                                       workspace, and the block that arrives last at such a node adds its
                                       partial rows in block order.  One launch, nothing to zero.  The library
                                       uses this flush by itself whenever the workspace has room for the
                                       partial rows (sized by gnn_workspace_bytes with max_dim >= dim; the
                                       size allows for blocks of >= 16 groups); with the flag a workspace
                                       without room is an error (GNN_EWORKSPACE) and the general kernel is
                                       always used.  Not combinable with GNN_FLAG_NO_BLOCK_OPT or
                                       GNN_FLAG_ATOMIC_FLUSH (GNN_EINVAL) */
#define GNN_FLAG_FUSION 64u         /* gnn_layer_forward / gnn_model_forward: fuse the Update GEMM into
                                       the aggregation kernel where the shape allows (out_dim <= 64, workspace
                                       with room for the ordered flush; in_dim of 16, 32 or 64 with groups of
                                       at most 4 x dw entries takes the wave-tile form, which ignores
                                       waves_per_block; other in_dim <= 128 that are multiples of 4 take the
                                       block-tile form with <= 8 waves per block, a multiple of
                                       ceil(out_dim/16)).  The library fuses by itself when the mean row has
                                       fewer than 8 entries (batches of small graphs: -20 % of a model pass)
                                       and either the wave-tile form applies or the layer's input is at most
                                       160 MB; on graphs with long rows the fused layer is as fast as the two
                                       separate kernels at best, hence the flag.  GNN_GCN: only a layer that
                                       aggregates first (out_dim > in_dim) can be fused, in the wave-tile form
                                       and only on request (measured slower than its two kernels) */
#define GNN_FLAG_NO_FUSION 512u     /* never fuse */
#define GNN_FLAG_ATOMIC_FLUSH 128u  /* always finish nodes that span blocks the way Sec. 5.2 describes: the
                                       leader adds the block's partial row to global memory with one float
                                       atomic per element (rows zeroed by a kernel that runs first, bias and
                                       activation of those rows by a kernel that runs last) */
#define GNN_FLAG_GCN_NARROW_FIRST 256u /* accepted and ignored: it asked for what is now the default (see below) */
#define GNN_FLAG_GCN_UPDATE_FIRST 1024u /* gnn_layer_forward / gnn_model_forward, GNN_GCN.  Sec. 3.1 orders the two
                                       phases of a GCN layer so that the aggregation runs at the smaller width:
                                       Update first when the layer narrows.  A layer whose output is wider than
                                       its input therefore aggregates first, at the input width, and updates
                                       afterwards: act((A_hat X) W + b) instead of act(A_hat (X W) + b), the same
                                       value up to rounding.  This flag keeps Update-then-Aggregation for such a
                                       layer too (the literal order of the paper's GCN) */

/* ================================================================================== */
/* HOST-side preparation                                                              */
/* ================================================================================== */

/* Community-aware node renumbering (Sec. 5.1).  HOST pointers; rowptr[n+1], colidx[nnz] a
 * symmetric CSR.  Computes AES (Eq. 4) and applies the rule sqrt(AES) > floor(sqrt(n)/100);
 * if it holds (or force != 0) clusters nodes by greedy modularity merging and numbers each
 * merge tree depth-first.  perm[old] = new, iperm[new] = old (both int32[n], caller-owned;
 * identity when no renumbering is done).  aes_out, did_reorder may be NULL.  Deterministic.
 * Errors: GNN_EINVAL (NULL, n < 0), GNN_ECSR (rowptr[0] != 0, decreasing, colidx out of range). */
int gnn_reorder(int32_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm,
                int32_t *iperm, double *aes_out, int *did_reorder, int force);

/* Eq. 4 alone: sum over stored entries of |row - col| and its mean.  HOST pointers. */
int gnn_aes(int32_t n, const int32_t *rowptr, const int32_t *colidx, int64_t *aes_sum, double *aes);

/* Eq. 2 weights: ew[e] = 1/sqrt(d_i * d_j) for entry e = (i, j), d = stored row length (the
 * CSR is expected to contain the self loops).  HOST pointers, ew float[nnz]. */
int gnn_gcn_norm(int32_t n, const int32_t *rowptr, const int32_t *colidx, float *ew);

/* Relabel a CSR by perm: row perm[i] of the result holds {perm[j]} ascending; val (may be
 * NULL together with val2) travels with its entry.  HOST pointers, outputs caller-owned with
 * the input's sizes. */
int gnn_apply_perm_csr(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *val,
                       const int32_t *perm, int32_t *rowptr2, int32_t *colidx2, float *val2);

/* Transpose of a CSR: entry (i, j, v) becomes (j, i, v); rows of the result sorted by column.  val /
 * val_t may both be NULL.  HOST pointers, outputs caller-owned with the input's sizes. */
int gnn_csr_transpose(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *val,
                      int32_t *rowptr_t, int32_t *colidx_t, float *val_t);

/* The parameter model re-derived for 256 CUs / 64-lane wavefronts / 160 KB LDS (Sec. 6).
 * Pure host function.  max_degree may be 0 (unknown).  ngs (neighbor-group size), dw (lanes that
 * share one neighbor row) and waves_per_block are IN/OUT: a positive value on entry is the caller's
 * choice and is kept, 0 asks for the model's choice given the others -- with max_degree = 0 exactly
 * what the DEVICE entry points do with their own ngs / dw / waves_per_block arguments (they cannot
 * read the longest row of a device CSR without synchronising).  The model's choices always fit the
 * scratch-memory limit of a block (see gnn_aggregate_gcn) for Dim up to 15,000.
 * Errors: GNN_EINVAL (NULL, negative, dw not a power of two <= 64, waves_per_block > 16). */
int gnn_decide(int32_t n, int64_t nnz, int32_t max_degree, int32_t dim, int32_t *ngs, int32_t *dw,
               int32_t *waves_per_block);

/* Eq. 5 and Eq. 6 exactly as printed, for reporting: dw from (dim, tpw); WPT = ngs*dim/dw;
 * SMEM = (tpb/tpw)*dim*4 bytes.  Any output may be NULL. */
int gnn_paper_model(int32_t dim, int32_t tpw, int32_t tpb, int32_t ngs, int32_t *dw, double *wpt,
                    int64_t *smem_bytes);

/* ================================================================================== */
/* DEVICE entry points                                                                */
/* ================================================================================== */

/* Bytes of DEVICE workspace (256-byte aligned) that the calls below need for a graph of n
 * nodes / nnz entries, neighbor-group size ngs (0 = whatever the model may pick) and, for
 * gnn_layer_forward, an intermediate of max_dim floats per node (0 for aggregation only).  The size
 * includes the scratch rows of GNN_FLAG_DETERMINISTIC for rows of up to max_dim floats. */
size_t gnn_workspace_bytes(int32_t n, int64_t nnz, int32_t max_dim, int32_t ngs);

/* Neighbor partitioning (Sec. 4.1): cuts every CSR row into groups of ngs consecutive entries
 * and stores, per group, (target node, start, end) in `workspace` -- the paper's
 * neighbor-partitioning graph store.  DEVICE rowptr.  One-time per (graph, ngs); later calls
 * pass GNN_FLAG_REUSE_PARTITION.  ngs >= 1. */
int gnn_partition_build(int32_t n, int64_t nnz, const int32_t *rowptr, int32_t ngs, void *workspace,
                        size_t workspace_bytes, void *stream);

/* Synchronises `stream` and reads the partition's status back: returns GNN_OK, or the error
 * the device kernels recorded (GNN_ECSR, GNN_ESTALE).  num_ng / ngs may be NULL. */
int gnn_workspace_status(const void *workspace, void *stream, int64_t *num_ng, int32_t *ngs);

/* Copies the stored neighbor groups to HOST arrays of `capacity` entries each (synchronises).
 * Returns GNN_ELIMIT if capacity < number of groups. */
int gnn_partition_export(const void *workspace, void *stream, int64_t capacity, int32_t *ng_node,
                         int32_t *ng_start, int32_t *ng_end);

/* Block layout of Algorithm 1 as the aggregation kernel derives it for (dw, waves_per_block):
 * per neighbor group its slot index inside its block and its leader flag, copied to HOST
 * arrays of `capacity` entries (synchronises).  groups_per_block (may be NULL) receives the
 * number of neighbor groups one block serves (Algorithm 1's warpPerBlock). */
int gnn_block_layout_export(const void *workspace, void *stream, int32_t dim, int32_t dw,
                            int32_t waves_per_block, int64_t capacity, int32_t *slot, uint8_t *leader,
                            int32_t *groups_per_block);

/* Checks a DEVICE CSR: rowptr[0] == 0, non-decreasing, rowptr[n] == nnz, 0 <= colidx < n.
 * Synchronises.  Returns GNN_OK or GNN_ECSR. */
int gnn_validate_csr_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                            void *stream);

/* GCN aggregation (Eq. 2 without the weight matrix): out = A_hat X with
 * out[i,:] = sum_{e in row i} ew[e] * X[colidx[e],:].  DEVICE pointers.  ew NULL = unit weights.
 * X, out: float[n*dim], out fully overwritten (rows without entries become 0).
 *   ngs  neighbor-group size, 0 = model's choice (Sec. 4.1, Sec. 6)
 *   dw   dimension workers: lanes sharing one neighbor row, a power of two <= 64, 0 = model's
 *        choice (Sec. 4.2); a wavefront serves 64/dw neighbor groups side by side
 *   waves_per_block  1..16, 0 = model's choice (the paper's user-chosen threads-per-block / 64)
 * Errors: GNN_EINVAL, GNN_EWORKSPACE, GNN_EHIP, and GNN_ELIMIT when a block's scratch memory would
 * exceed 64 KB: with T = waves_per_block * 64 / dw groups per block the need is
 *   round_up_16(4 * (T * ngs + 8) * (ew ? 2 : 1)) + 4 * waves_per_block * dim + 128 + 256 * waves_per_block  bytes
 * (the model's own choices never exceed it; caller-chosen ngs / dw / waves_per_block can). */
int gnn_aggregate_gcn(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                      const float *ew, const float *X, float *out, int32_t dim, int32_t ngs,
                      int32_t dw, int32_t waves_per_block, uint32_t flags, void *workspace,
                      size_t workspace_bytes, void *stream);

/* GIN aggregation (the argument of h in Eq. 3): out[i,:] = (1+eps) X[i,:] + sum_{j in N(i)} X[j,:].
 * The CSR holds no self loops.  Other arguments as above. */
int gnn_aggregate_gin(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float eps,
                      const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw,
                      int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                      void *stream);

/* gnn_aggregate_gin for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same
 * kernels, same arguments, but the neighbor partition, the arrival counters and the partial rows of
 * the ordered flush live in a fixed array of 128 MiB of device memory inside the library (one per GPU,
 * held until the process ends) instead of a caller's workspace.  The call allocates nothing.
 *   Limit: gnn_workspace_bytes(n, nnz, dim, ngs) must not exceed 128 MiB (ngs = 0: the model's choice;
 *   e.g. 1 M nodes / 16 M entries at dim 64 need 81 MB), else GNN_ELIMIT and nothing is enqueued.
 *   Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 *   threads) race; calls on one stream are ordered.  The array keeps the last call's partition, so
 *   GNN_FLAG_REUSE_PARTITION is honoured for a repeated (rowptr, n, nnz, ngs) and reports GNN_ESTALE
 *   otherwise; without the flag the partition is built (and the counters cleared) by kernels of this call.
 *   scratch_out (HOST, may be NULL) receives the DEVICE address of the array, for gnn_workspace_status
 *   and gnn_partition_export.
 * Errors: as gnn_aggregate_gin, and GNN_ELIMIT as above. */
int gnn_aggregate_gin_static(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float eps,
                             const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw,
                             int32_t waves_per_block, uint32_t flags, void *stream, void **scratch_out);

/* Aggregation over the neighbour embeddings alone with another reduction (Sec. 3.1 names sum and
 * min as examples): out[i,:] = reduce over the stored entries j of row i of X[j,:], no weights, no
 * self term.  op: GNN_REDUCE_SUM, GNN_REDUCE_MAX, GNN_REDUCE_MIN (elementwise, exact) or
 * GNN_REDUCE_MEAN (sum divided by the row length).  A row without entries gives 0.  Max, min and mean
 * use the ordered flush, so the workspace must be sized with max_dim >= dim (GNN_EWORKSPACE otherwise)
 * and the flags GNN_FLAG_NO_BLOCK_OPT, _ATOMIC_FLUSH, _FUSION are refused (GNN_EINVAL).
 * Everything else as for gnn_aggregate_gcn. */
#define GNN_REDUCE_SUM 0
#define GNN_REDUCE_MAX 1
#define GNN_REDUCE_MIN 2
#define GNN_REDUCE_MEAN 3
int gnn_aggregate_reduce(int op, int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                         const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw,
                         int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                         void *stream);

/* Aggregation with a feature vector on every stored entry (Sec. 3.1: the second class of aggregation applies
 * edge features to each neighbor; the paper does not fix the combination, the reading here is the
 * elementwise product): out[i,:] = sum over the stored entries e = (i, j) of row i of E[e,:] * X[j,:].
 * E: DEVICE float[nnz, dim], one row per stored entry in CSR order, read once.  No scalar weights, no self
 * term; a row without entries gives 0.  Scalar edge weights go through the ew argument of
 * gnn_aggregate_gcn instead.  Uses the ordered flush, so the workspace must be sized with max_dim >= dim
 * (GNN_EWORKSPACE otherwise) and the flags GNN_FLAG_NO_BLOCK_OPT, _ATOMIC_FLUSH, _FUSION are refused
 * (GNN_EINVAL).  Everything else as for gnn_aggregate_gcn. */
int gnn_aggregate_edge(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *E,
                       const float *X, float *out, int32_t dim, int32_t ngs, int32_t dw,
                       int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                       void *stream);

/* Update phase alone (Sec. 2.1, w.a + b): out[n,M] = act(A[n,K] W[K,M] + b), fp32 MFMA.
 * b NULL or float[M]; relu 0/1.  DEVICE pointers. */
int gnn_update_gemm(int32_t n, int32_t K, int32_t M, const float *A, const float *W, const float *b,
                    int relu, float *out, void *stream);

/* One GNN layer (Eq. 1).  kind GNN_GCN: out = act(A_hat (X W) + b), computed as Update then
 * Aggregation when out_dim <= in_dim and as act((A_hat X) W + b), Aggregation then Update, when the layer
 * widens (Sec. 3.1: the aggregation runs at the smaller width; GNN_FLAG_GCN_UPDATE_FIRST keeps the first
 * order);  GNN_GIN: out = act(((1+eps) X + sum_N X) W + b).  X float[n*in_dim], W float[in_dim*out_dim]
 * row-major, b NULL or float[out_dim], out float[n*out_dim].  The intermediate lives in the workspace
 * (size it with max_dim = max(in_dim, out_dim)).  ew is used by GNN_GCN only, eps by GNN_GIN only. */
int gnn_layer_forward(int kind, int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                      const float *ew, float eps, const float *X, int32_t in_dim, const float *W,
                      const float *b, int32_t out_dim, int relu, float *out, int32_t ngs, int32_t dw,
                      int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                      void *stream);

/* A whole model in one call (the evaluation settings of Sec. 7.1: GCN 2 layers, GIN 5 layers):
 * num_layers calls of gnn_layer_forward chained, ReLU after every layer but the last, the neighbor
 * partition built once (or reused with GNN_FLAG_REUSE_PARTITION).  dims: HOST int32[num_layers+1],
 * layer l maps dims[l] -> dims[l+1].  W: HOST array of num_layers DEVICE pointers (W[l] is
 * float[dims[l]*dims[l+1]]); b: NULL, or a HOST array of num_layers DEVICE pointers or NULLs.
 * X float[n*dims[0]], out float[n*dims[num_layers]] (DEVICE).  The hidden activations live in the
 * workspace, which gnn_model_workspace_bytes sizes (layer workspace + two activation buffers).
 * ev_agg_start / ev_agg_stop: NULL, or HOST arrays of num_layers hipEvent_t (entries may be NULL)
 * recorded around the aggregation kernel of each layer, as in gnn_layer_forward_timed.
 * Only enqueues; the host arrays are read before the call returns. */
size_t gnn_model_workspace_bytes(int32_t n, int64_t nnz, int32_t num_layers, const int32_t *dims, int32_t ngs);
int gnn_model_forward(int kind, int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                      const float *ew, float eps, const float *X, int32_t num_layers, const int32_t *dims,
                      const float *const *W, const float *const *b, float *out, int32_t ngs, int32_t dw,
                      int32_t waves_per_block, uint32_t flags, void *workspace, size_t workspace_bytes,
                      void *stream, void *const *ev_agg_start, void *const *ev_agg_stop);

/* Backward pass of gnn_layer_forward (training; the aggregation kernel is reused on gradients,
 * Sec. 7.2).  rowptr_t / colidx_t / ew_t: the TRANSPOSED graph (gnn_csr_transpose; a symmetric graph
 * with symmetric weights is its own transpose), and `workspace` holds ITS partition.
 *   kind GNN_GCN: forward was Y = act(A_hat (X W) + b);  P = X float[n*in_dim].
 *                 dW = X^T (A_hat^T dZ),  dX = (A_hat^T dZ) W^T,  dZ = dY masked by Y > 0 when relu.
 *   kind GNN_GIN: forward was Y = act(A W + b), A = (1+eps) X + sum_N X;  P = A float[n*in_dim]
 *                 (the caller keeps A from gnn_aggregate_gin).  dW = A^T dZ,  dX = (1+eps) dA + sum over
 *                 the transposed graph of dA,  dA = dZ W^T.
 * Y (forward output, needed only when relu), dY: float[n*out_dim].  Outputs: dW float[in_dim*out_dim],
 * db float[out_dim] or NULL, dX float[n*in_dim] or NULL (first layer).  Workspace of
 * gnn_backward_workspace_bytes().  DEVICE pointers; only enqueues. */
size_t gnn_backward_workspace_bytes(int32_t n, int64_t nnz, int32_t in_dim, int32_t out_dim, int32_t ngs);
int gnn_layer_backward(int kind, int32_t n, int64_t nnz, const int32_t *rowptr_t, const int32_t *colidx_t,
                       const float *ew_t, float eps, const float *P, int32_t in_dim, const float *W,
                       int32_t out_dim, int relu, const float *Y, const float *dY, float *dX, float *dW,
                       float *db, int32_t ngs, int32_t dw, int32_t waves_per_block, uint32_t flags,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Graph preparation on the DEVICE (one-time per graph; these three allocate their own temporaries
 * with hipMalloc and, except gnn_gcn_norm_device, synchronise `stream` before they return).
 *
 * gnn_reorder_device: the community renumbering of Sec. 5.1 with a round-based merge schedule (all
 * communities act on the same state in synchronous rounds: propose to the neighbouring community of
 * largest modularity gain, the smaller id of a mutual pair stays, only proposals to a community that
 * does not move itself are carried out, joiners are appended by ascending id; new ids = communities
 * by ascending root id, then position).  The permutation differs from gnn_reorder's (another merge
 * schedule) and gives about the same locality at a small fraction of the time.  DEVICE rowptr[n+1],
 * colidx[nnz] (symmetric CSR, validated), DEVICE perm[n], iperm[n].  max_rounds bounds the rounds (64
 * is ample); rounds_out (HOST, may be NULL) receives the rounds that merged something.  No AES rule
 * here: call gnn_aes / decide on the host if wanted.  Deterministic (integer arithmetic only).
 * Errors: GNN_EINVAL, GNN_ECSR (column index out of range), GNN_EHIP.
 *
 * gnn_apply_perm_csr_device: gnn_apply_perm_csr on DEVICE arrays, same result byte for byte.
 * Errors: GNN_EINVAL (perm not a bijection), GNN_ECSR, GNN_EHIP.
 *
 * gnn_csr_transpose_device: gnn_csr_transpose on DEVICE arrays (the graph gnn_layer_backward wants),
 * same result byte for byte.  Errors: GNN_EINVAL, GNN_ECSR, GNN_EHIP.
 *
 * gnn_gcn_norm_device: gnn_gcn_norm on DEVICE arrays, same result byte for byte; only enqueues.
 *
 * gnn_aes_device: Eq. 4 and the rule of Sec. 5.1 on a DEVICE CSR (what gnn_aes and the decision inside
 * gnn_reorder compute on the host).  aes_sum, aes, should_reorder are HOST outputs, any may be NULL. */
int gnn_reorder_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, int32_t *perm,
                       int32_t *iperm, int32_t max_rounds, int32_t *rounds_out, void *stream);
int gnn_apply_perm_csr_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                              const int32_t *perm, int32_t *rowptr2, int32_t *colidx2, float *val2, void *stream);
int gnn_csr_transpose_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                             int32_t *rowptr_t, int32_t *colidx_t, float *val_t, void *stream);
int gnn_gcn_norm_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, float *ew, void *stream);
int gnn_aes_device(int32_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, int64_t *aes_sum, double *aes,
                   int *should_reorder, void *stream);

/* Row gather for renumbering: Y[perm[i],:] = X[i,:] (pass iperm to undo).  DEVICE pointers,
 * perm int32[n]. */
int gnn_permute_rows(int32_t n, int32_t dim, const int32_t *perm, const float *X, float *Y, void *stream);

/* ---- diagnostics ------------------------------------------------------------------ */
const char *gnn_strerror(int code);
int gnn_last_hip_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int gnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GNN_MI355X_H */
