/*
 * CPU oracle for the GNN aggregation path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C.  It defines what the GPU library must compute
 * and is compared with it element by element; it is never a fallback for it.
 * Only the tests, the smoke check and the benchmark's "cpu_baseline" leg load it.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Floating point: every sum is accumulated in double and rounded to float once,
 * when the result of an operation (aggregation, dense layer) is stored.  Values
 * between operations are float, as they are on the GPU.
 *
 * Pins (tests/test_oracle_*.py, all run without a GPU), function by function:
 *   orc_aggregate_gcn     aggregate.py: gcn_matches_dense_product, gcn_is_not_symmetric_in_its_operands,
 *                         all_ones_features_give_normalised_degree_sums, regular_graph_..._to_one,
 *                         star_graph_closed_form, linearity_and_eps_term, empty_graph_and_isolated_nodes,
 *                         oracle_against_a_library_sparse_product; abs_out: layers.py:
 *                         aggregation_error_scales_are_the_sums_of_absolute_terms
 *   orc_aggregate_edge_vec edge_vec.py: matches_the_dense_tensor_expression, constant_vectors_reduce_to_the_weighted_sum,
 *                         one_hot_vectors_select_single_dimensions, hand_worked_triangle, renumbering_invariance
 *   orc_aggregate_f64     layers.py: gcn_layer_error_scale_equals_the_dense_expression
 *   orc_aggregate_gin     aggregate.py: gin_matches_dense_product, all_ones..., linearity_and_eps_term,
 *                         empty_graph_and_isolated_nodes; abs_out as above
 *   orc_aggregate_reduce  reduce.py: reductions_match_numpy_over_explicit_neighbour_lists,
 *                         closed_forms_on_a_path_and_a_star, order_relations_and_link_to_the_sum_aggregation
 *   orc_gemm_bias_act     aggregate.py: gemm_matches_numpy, gemm_identity_and_non_square_orientation;
 *                         abs_out: layers.py as above
 *   orc_bias_act          layers.py: bias_act_values_worked_by_hand, bias_is_broadcast_over_rows_not_columns,
 *                         gcn_layer_with_bias_equals_the_dense_expression
 *   orc_gcn_norm          aggregate.py: gcn_norm_is_symmetric_bitwise, regular graph -> 1/(k+1), star
 *   orc_aes_sum, orc_aes_threshold, orc_should_reorder
 *                         structure.py: aes_hand_computed, aes_thresholds_from_the_rule
 *   orc_ng_partition      structure.py: paper_worked_example_of_neighbor_groups (tests/golden/
 *                         ng_partition_example.txt), neighbor_groups_tile_the_csr
 *   orc_alg1_layout       structure.py: alg1_hand_trace (tests/golden/alg1_trace.txt), alg1_invariants,
 *                         global_flushes_per_block_are_bounded
 *   orc_eq5_*, orc_eq6_dw structure.py: eq5_eq6_literal_values
 *   orc_reorder           structure.py: reorder_hand_trace (tests/golden/reorder_trace.txt),
 *                         reorder_is_a_bijection_and_deterministic, ..._interleaved_cliques_contiguous,
 *                         ..._lowers_aes_of_shuffled_block_diagonal_batch, ..._finds_planted_communities,
 *                         ..._path_graph_keeps_small_span
 *   orc_apply_perm_csr, orc_permute_rows
 *                         structure.py: apply_perm_csr_and_permute_rows,
 *                         renumbering_leaves_the_aggregation_unchanged
 * The compositions in __init__.py (gcn_layer, gin_layer, gcn_model, gin_model, their error scales,
 * the backward pass) are pinned by tests/test_oracle_layers.py (dense double-precision expressions,
 * bias after the aggregation, ReLU after every layer but the last) and tests/test_oracle_backward.py
 * (finite differences); parallel_reorder.py by tests/test_oracle_parallel_reorder.py.
 * Parity unpinned: none of the functions below.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ Eq. 2: GCN aggregation
 * out[i,:] = sum over stored entries e of row i of ew[e] * X[colidx[e],:].
 * The matrix D^-1/2 A D^-1/2 is handed in as CSR structure + ew (see orc_gcn_norm);
 * ew == NULL means unit weights.  abs_out (may be NULL) receives sum |ew * x|, the
 * scale against which a floating-point sum in any order may be judged. */
void orc_aggregate_gcn(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *ew,
                       const float *X, int32_t dim, float *out, double *abs_out)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t k = 0; k < dim; ++k) {
            double acc = 0.0, aacc = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double w = ew ? (double)ew[e] : 1.0;
                double t = w * (double)X[(size_t)colidx[e] * dim + k];
                acc += t;
                aacc += fabs(t);
            }
            out[(size_t)i * dim + k] = (float)acc;
            if (abs_out) abs_out[(size_t)i * dim + k] = aacc;
        }
    }
}

/* Aggregation with a feature vector on every stored entry (Sec. 3.1, the second class of aggregation:
 * edge features applied to each neighbor): out[i,k] = sum over stored entries e of row i of
 * E[e,k] * X[colidx[e],k].  E holds one row of dim floats per stored entry, in CSR order.  A vector whose
 * dim entries all equal a scalar w[e] gives orc_aggregate_gcn with the weights w. */
void orc_aggregate_edge_vec(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *E,
                            const float *X, int32_t dim, float *out, double *abs_out)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t k = 0; k < dim; ++k) {
            double acc = 0.0, aacc = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double t = (double)E[(size_t)e * dim + k] * (double)X[(size_t)colidx[e] * dim + k];
                acc += t;
                aacc += fabs(t);
            }
            out[(size_t)i * dim + k] = (float)acc;
            if (abs_out) abs_out[(size_t)i * dim + k] = aacc;
        }
    }
}

/* The same sum over doubles: out[i,:] = sum over stored entries e of row i of w[e] * X[colidx[e],:]
 * (w NULL = unit weights), nothing rounded to float.  Used for the error scale of a GCN layer,
 * |A_hat| (|X| |W|), whose inner factor is already a double. */
void orc_aggregate_f64(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w,
                       const double *X, int32_t dim, double *out)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t k = 0; k < dim; ++k) {
            double acc = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                acc += (w ? w[e] : 1.0) * X[(size_t)colidx[e] * dim + k];
            out[(size_t)i * dim + k] = acc;
        }
    }
}

/* ------------------------------------------------------------------ Eq. 3: GIN aggregation
 * out[i,:] = (1 + eps) * X[i,:] + sum_{j in N(i)} X[j,:]   (the argument of h in Eq. 3). */
void orc_aggregate_gin_rows(int32_t row_begin, int32_t row_end, const int32_t *rowptr, const int32_t *colidx,
                            float eps, const float *X, int32_t dim, float *out, double *abs_out)
{
    for (int32_t i = row_begin; i < row_end; ++i) {
        for (int32_t k = 0; k < dim; ++k) {
            double self = (1.0 + (double)eps) * (double)X[(size_t)i * dim + k];
            double acc = self, aacc = fabs(self);
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double t = (double)X[(size_t)colidx[e] * dim + k];
                acc += t;
                aacc += fabs(t);
            }
            out[(size_t)i * dim + k] = (float)acc;
            if (abs_out) abs_out[(size_t)i * dim + k] = aacc;
        }
    }
}

/* All rows.  (The row-range form above exists so that the benchmark's all-cores baseline can hand
 * disjoint row ranges of the same loop to several threads; rows are independent.) */
void orc_aggregate_gin(int32_t n, const int32_t *rowptr, const int32_t *colidx, float eps,
                       const float *X, int32_t dim, float *out, double *abs_out)
{
    orc_aggregate_gin_rows(0, n, rowptr, colidx, eps, X, dim, out, abs_out);
}

/* ------------------------------------------------------------------ Sec. 3.1: other neighbour aggregations
 * The paper names sum and min as examples of aggregation over the neighbour embeddings only; mean
 * and max are the other two reductions GNN layers use.  No self term, no weights.
 * op 1: out[i,k] = max_j X[j,k];  op 2: min;  op 3: mean = (sum_j X[j,k]) / deg(i), summed in double.
 * A row without entries gives 0 (there is nothing to reduce; 0 is what a sum gives).  Duplicate
 * entries count as often as they are stored (mean), and do not matter for max/min.
 * abs_out (op 3 only, may be NULL): sum |x| / deg, the error scale of the mean. */
void orc_aggregate_reduce(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *X, int32_t dim,
                          int32_t op, float *out, double *abs_out)
{
    for (int32_t i = 0; i < n; ++i) {
        const int32_t deg = rowptr[i + 1] - rowptr[i];
        for (int32_t k = 0; k < dim; ++k) {
            float best = 0.0f;
            double acc = 0.0, aacc = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const float x = X[(size_t)colidx[e] * dim + k];
                if (e == rowptr[i]) best = x;
                else if (op == 1 && x > best) best = x;
                else if (op == 2 && x < best) best = x;
                acc += (double)x;
                aacc += fabs((double)x);
            }
            float r = best;
            if (op == 3) r = deg > 0 ? (float)(acc / (double)deg) : 0.0f;
            out[(size_t)i * dim + k] = r;
            if (abs_out) abs_out[(size_t)i * dim + k] = deg > 0 ? aacc / (double)deg : 0.0;
        }
    }
}

/* ------------------------------------------------------------------ Sec. 2.1: Update, w.a + b
 * out[i,m] = act( b[m] + sum_k A[i,k] * W[k,m] ),  A[n,K], W[K,M] row-major, b NULL or [M]. */
void orc_gemm_bias_act(int32_t n, int32_t K, int32_t M, const float *A, const float *W,
                       const float *b, int32_t relu, float *out, double *abs_out)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t m = 0; m < M; ++m) {
            double acc = b ? (double)b[m] : 0.0;
            double aacc = fabs(acc);
            for (int32_t k = 0; k < K; ++k) {
                double t = (double)A[(size_t)i * K + k] * (double)W[(size_t)k * M + m];
                acc += t;
                aacc += fabs(t);
            }
            if (relu && acc < 0.0) acc = 0.0;
            out[(size_t)i * M + m] = (float)acc;
            if (abs_out) abs_out[(size_t)i * M + m] = aacc;
        }
    }
}

/* out = act(in + b) row-wise: the bias/activation that follows a GCN aggregation. */
void orc_bias_act(int32_t n, int32_t M, const float *in, const float *b, int32_t relu, float *out)
{
    for (int32_t i = 0; i < n; ++i)
        for (int32_t m = 0; m < M; ++m) {
            float v = in[(size_t)i * M + m];
            if (b) v = (float)((double)v + (double)b[m]);
            if (relu && v < 0.0f) v = 0.0f;
            out[(size_t)i * M + m] = v;
        }
}

/* ------------------------------------------------------------------ Eq. 2: D^-1/2 A D^-1/2
 * ew[e] = 1 / sqrt(d_i * d_j) for entry e = (i, j), d = stored row length (the CSR already
 * contains the self loops). */
void orc_gcn_norm(int32_t n, const int32_t *rowptr, const int32_t *colidx, float *ew)
{
    for (int32_t i = 0; i < n; ++i) {
        double di = (double)(rowptr[i + 1] - rowptr[i]);
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int32_t j = colidx[e];
            double dj = (double)(rowptr[j + 1] - rowptr[j]);
            ew[e] = (float)(1.0 / sqrt(di * dj));
        }
    }
}

/* ------------------------------------------------------------------ Eq. 4: averaged edge span
 * Returns sum |src - trg| over all stored entries (AES = that / nnz). */
int64_t orc_aes_sum(int32_t n, const int32_t *rowptr, const int32_t *colidx)
{
    int64_t s = 0;
    for (int32_t i = 0; i < n; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int64_t d = (int64_t)i - (int64_t)colidx[e];
            s += d < 0 ? -d : d;
        }
    return s;
}

/* Sec. 5.1 rule: renumber when sqrt(AES) > floor(sqrt(N)/100).  Both sides are >= 0, so the
 * test is AES > T^2 with T = floor(sqrt(N)/100), i.e. aes_sum > T^2 * nnz, in integers. */
int32_t orc_aes_threshold(int32_t n)
{
    int64_t r = (int64_t)floor(sqrt((double)n));
    while (r * r > (int64_t)n) --r;
    while ((r + 1) * (r + 1) <= (int64_t)n) ++r;
    return (int32_t)(r / 100);
}

int32_t orc_should_reorder(int32_t n, int64_t nnz, int64_t aes_sum)
{
    int64_t T = orc_aes_threshold(n);
    return aes_sum > T * T * nnz ? 1 : 0;
}

/* ------------------------------------------------------------------ Sec. 4.1: neighbor partitioning
 * Cuts every row of the CSR into groups of ngs consecutive entries (the last group of a row may
 * be shorter); a group never spans two rows.  Group g has target node ng_node[g] and covers CSR
 * positions [ng_start[g], ng_end[g]).  Returns the number of groups; arrays may be NULL to count. */
int64_t orc_ng_partition(int32_t n, const int32_t *rowptr, int32_t ngs,
                         int32_t *ng_node, int32_t *ng_start, int32_t *ng_end)
{
    int64_t g = 0;
    for (int32_t v = 0; v < n; ++v) {
        for (int32_t s = rowptr[v]; s < rowptr[v + 1]; s += ngs) {
            int32_t e = s + ngs < rowptr[v + 1] ? s + ngs : rowptr[v + 1];
            if (ng_node) {
                ng_node[g] = v;
                ng_start[g] = s;
                ng_end[g] = e;
            }
            ++g;
        }
    }
    return g;
}

/* ------------------------------------------------------------------ Algorithm 1
 * What the algorithm assigns, stated as a definition.  Workers (one per neighbor group; the paper's
 * "warps") are cut into blocks of warpPerBlock consecutive workers.  Inside a block the workers of
 * one target node are consecutive (groups are stored node by node), so the block's distinct target
 * nodes can be numbered 0, 1, 2, ... in the order in which they first appear:
 *   slot[g]   = that number for the target node of worker g: the node's slot in the block's scratch
 *               memory; its float offset is sharedAddr[g] = slot[g] * Dim (the printed algorithm
 *               mixes index and offset; the offset reading is used throughout);
 *   leader[g] = 1 for the first worker of each (block, node) pair, else 0: the one worker that
 *               moves the slot to global memory. */
void orc_alg1_layout(int64_t warpNum, const int32_t *nodeID, int32_t warpPerBlock, int32_t Dim,
                     int32_t *slot, int64_t *sharedAddr, uint8_t *leader)
{
    for (int64_t block_first = 0; block_first < warpNum; block_first += warpPerBlock) {
        int64_t block_end = block_first + warpPerBlock < warpNum ? block_first + warpPerBlock : warpNum;
        int32_t distinct = 0; /* target nodes seen so far in this block */
        for (int64_t g = block_first; g < block_end; ++g) {
            int opens_node = (g == block_first) || (nodeID[g] != nodeID[g - 1]);
            if (opens_node) ++distinct;
            slot[g] = distinct - 1;
            sharedAddr[g] = (int64_t)slot[g] * Dim;
            leader[g] = opens_node ? 1 : 0;
        }
    }
}

/* ------------------------------------------------------------------ Eq. 5 and Eq. 6 (as printed) */
double orc_eq5_wpt(int32_t ngs, int32_t Dim, int32_t dw) { return (double)ngs * (double)Dim / (double)dw; }
int64_t orc_eq5_smem(int32_t tpb, int32_t tpw, int32_t Dim) { return (int64_t)(tpb / tpw) * Dim * 4; }
int32_t orc_eq6_dw(int32_t Dim, int32_t tpw) { return Dim >= tpw ? tpw : tpw / 2; }

/* ------------------------------------------------------------------ Sec. 5.1: community-aware renumbering
 *
 * The paper names the method (merge vertices greedily by modularity gain, then number every
 * cluster by a depth-first walk of its merge tree) without fixing details; the reading below is
 * this build's deterministic, integer-only one.  The library implements the same reading with
 * different data structures; results must agree byte for byte.
 *
 *  1. Clean adjacency: per vertex the set of distinct neighbours other than itself, unit weights.
 *     deg0[v] = its size, M2 = sum deg0.  Every vertex starts as its own cluster, degw = deg0.
 *  2. Visit vertices in ascending (deg0, id).  At the visit of u, collect its cluster's edges:
 *     u's own clean list plus, for every child c merged into u so far (in merge order), the list
 *     c stored when it was visited.  Map every endpoint to its current root, drop u itself, add up
 *     the weights per root.  Score S(v) = w(u,v) * M2 - degw[u] * degw[v]  (the sign and order of the
 *     modularity gain of merging u into v).  Take the largest S, ties to the smallest v.  If it is
 *     > 0: parent[u] = v, degw[v] += degw[u], u is appended to v's children, and u keeps its
 *     collected list for v's later visit.  Otherwise u stays a top-level root.
 *  3. New ids: top-level roots in ascending id; each root's merge tree in depth-first pre-order,
 *     children in merge order.  perm[old] = new, iperm[new] = old.
 */
typedef struct { int32_t v; int64_t w; } orc_pair;

static int orc_pair_cmp(const void *a, const void *b)
{
    int32_t x = ((const orc_pair *)a)->v, y = ((const orc_pair *)b)->v;
    return x < y ? -1 : (x > y ? 1 : 0);
}

static int32_t orc_root(const int32_t *parent, int32_t x)
{
    while (parent[x] != x) x = parent[x];
    return x;
}

static int orc_i32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

int32_t orc_reorder(int32_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm, int32_t *iperm)
{
    if (n <= 0) return 0;
    /* step 1: clean adjacency */
    int64_t *cptr = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    int32_t *cadj = (int32_t *)malloc(sizeof(int32_t) * (size_t)(rowptr[n] > 0 ? rowptr[n] : 1));
    int32_t *tmp = NULL;
    int32_t tmpcap = 0;
    int64_t M2 = 0;
    for (int32_t i = 0; i < n; ++i) {
        int32_t len = rowptr[i + 1] - rowptr[i];
        if (len > tmpcap) { tmpcap = len * 2; tmp = (int32_t *)realloc(tmp, sizeof(int32_t) * (size_t)tmpcap); }
        for (int32_t k = 0; k < len; ++k) tmp[k] = colidx[rowptr[i] + k];
        qsort(tmp, (size_t)len, sizeof(int32_t), orc_i32_cmp);
        cptr[i] = M2;
        for (int32_t k = 0; k < len; ++k) {
            if (tmp[k] == i) continue;
            if (k > 0 && tmp[k] == tmp[k - 1]) continue;
            cadj[M2++] = tmp[k];
        }
    }
    cptr[n] = M2;
    free(tmp);

    /* visiting order: ascending (deg0, id) */
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    {
        int64_t maxd = 0;
        for (int32_t i = 0; i < n; ++i) { int64_t d = cptr[i + 1] - cptr[i]; if (d > maxd) maxd = d; }
        int64_t *bucket = (int64_t *)calloc((size_t)maxd + 2, sizeof(int64_t));
        for (int32_t i = 0; i < n; ++i) bucket[cptr[i + 1] - cptr[i] + 1]++;
        for (int64_t d = 0; d <= maxd; ++d) bucket[d + 1] += bucket[d];
        for (int32_t i = 0; i < n; ++i) order[bucket[cptr[i + 1] - cptr[i]]++] = i;
        free(bucket);
    }

    int32_t *parent = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int64_t *degw = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
    /* children as linked lists in merge order */
    int32_t *first_child = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *last_child = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *next_sib = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    orc_pair **stored = (orc_pair **)calloc((size_t)n, sizeof(orc_pair *));
    int64_t *stored_len = (int64_t *)calloc((size_t)n, sizeof(int64_t));
    for (int32_t i = 0; i < n; ++i) {
        parent[i] = i;
        degw[i] = cptr[i + 1] - cptr[i];
        first_child[i] = last_child[i] = next_sib[i] = -1;
    }

    orc_pair *buf = NULL;
    int64_t bufcap = 0;
    for (int32_t oi = 0; oi < n; ++oi) {
        int32_t u = order[oi];
        /* step 2: collect */
        int64_t need = cptr[u + 1] - cptr[u];
        for (int32_t c = first_child[u]; c >= 0; c = next_sib[c]) need += stored_len[c];
        if (need > bufcap) { bufcap = need * 2 + 16; buf = (orc_pair *)realloc(buf, sizeof(orc_pair) * (size_t)bufcap); }
        int64_t m = 0;
        for (int64_t k = cptr[u]; k < cptr[u + 1]; ++k) {
            int32_t r = orc_root(parent, cadj[k]);
            if (r != u) { buf[m].v = r; buf[m].w = 1; ++m; }
        }
        for (int32_t c = first_child[u]; c >= 0; c = next_sib[c]) {
            for (int64_t k = 0; k < stored_len[c]; ++k) {
                int32_t r = orc_root(parent, stored[c][k].v);
                if (r != u) { buf[m].v = r; buf[m].w = stored[c][k].w; ++m; }
            }
            free(stored[c]);
            stored[c] = NULL;
            stored_len[c] = 0;
        }
        qsort(buf, (size_t)m, sizeof(orc_pair), orc_pair_cmp);
        int64_t u_len = 0;
        for (int64_t k = 0; k < m; ++k) {
            if (u_len > 0 && buf[u_len - 1].v == buf[k].v) buf[u_len - 1].w += buf[k].w;
            else buf[u_len++] = buf[k];
        }
        /* score; buf is sorted by v, so the first maximum is the smallest v */
        int32_t best = -1;
        int64_t bestS = 0;
        for (int64_t k = 0; k < u_len; ++k) {
            int64_t S = buf[k].w * M2 - degw[u] * degw[buf[k].v];
            if (best < 0 || S > bestS) { best = buf[k].v; bestS = S; }
        }
        if (best >= 0 && bestS > 0) {
            parent[u] = best;
            degw[best] += degw[u];
            if (last_child[best] < 0) first_child[best] = u; else next_sib[last_child[best]] = u;
            last_child[best] = u;
            stored[u] = (orc_pair *)malloc(sizeof(orc_pair) * (size_t)(u_len > 0 ? u_len : 1));
            memcpy(stored[u], buf, sizeof(orc_pair) * (size_t)u_len);
            stored_len[u] = u_len;
        }
    }

    /* step 3: depth-first pre-order over the merge forest */
    int32_t *stack = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t next_id = 0;
    for (int32_t r = 0; r < n; ++r) {
        if (parent[r] != r) continue;
        int32_t sp = 0;
        stack[sp++] = r;
        while (sp > 0) {
            int32_t x = stack[--sp];
            perm[x] = next_id;
            iperm[next_id] = x;
            ++next_id;
            /* push children in reverse merge order so that the first merged is numbered first */
            int32_t cnt = 0;
            for (int32_t c = first_child[x]; c >= 0; c = next_sib[c]) { stack[sp + cnt] = c; ++cnt; }
            for (int32_t a = 0, b = cnt - 1; a < b; ++a, --b) {
                int32_t t = stack[sp + a]; stack[sp + a] = stack[sp + b]; stack[sp + b] = t;
            }
            sp += cnt;
        }
    }
    for (int32_t i = 0; i < n; ++i) if (stored[i]) free(stored[i]);
    free(stack); free(buf); free(stored); free(stored_len);
    free(first_child); free(last_child); free(next_sib);
    free(parent); free(degw); free(order); free(cptr); free(cadj);
    return next_id == n ? 0 : -1;
}

/* Relabel a CSR: row perm[i] of the result holds {perm[j]} in ascending order; per-entry values
 * val (may be NULL) travel with their entry. */
typedef struct { int32_t c; float v; } orc_cv;
static int orc_cv_cmp(const void *a, const void *b)
{
    int32_t x = ((const orc_cv *)a)->c, y = ((const orc_cv *)b)->c;
    return x < y ? -1 : (x > y ? 1 : 0);
}

void orc_apply_perm_csr(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *val,
                        const int32_t *perm, int32_t *rowptr2, int32_t *colidx2, float *val2)
{
    int32_t *iperm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int32_t i = 0; i < n; ++i) iperm[perm[i]] = i;
    rowptr2[0] = 0;
    for (int32_t r = 0; r < n; ++r) {
        int32_t i = iperm[r];
        rowptr2[r + 1] = rowptr2[r] + (rowptr[i + 1] - rowptr[i]);
    }
    int32_t cap = 16;
    orc_cv *row = (orc_cv *)malloc(sizeof(orc_cv) * (size_t)cap);
    for (int32_t r = 0; r < n; ++r) {
        int32_t i = iperm[r];
        int32_t len = rowptr[i + 1] - rowptr[i];
        if (len > cap) { cap = len * 2; row = (orc_cv *)realloc(row, sizeof(orc_cv) * (size_t)cap); }
        for (int32_t k = 0; k < len; ++k) {
            row[k].c = perm[colidx[rowptr[i] + k]];
            row[k].v = val ? val[rowptr[i] + k] : 0.0f;
        }
        qsort(row, (size_t)len, sizeof(orc_cv), orc_cv_cmp);
        for (int32_t k = 0; k < len; ++k) {
            colidx2[rowptr2[r] + k] = row[k].c;
            if (val2) val2[rowptr2[r] + k] = row[k].v;
        }
    }
    free(row);
    free(iperm);
}

/* Rows of X moved to their new position: Y[perm[i],:] = X[i,:]. */
void orc_permute_rows(int32_t n, int32_t dim, const int32_t *perm, const float *X, float *Y)
{
    for (int32_t i = 0; i < n; ++i)
        memcpy(Y + (size_t)perm[i] * dim, X + (size_t)i * dim, sizeof(float) * (size_t)dim);
}
