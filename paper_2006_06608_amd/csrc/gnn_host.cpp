// Host-side preparation: renumbering (Sec. 5.1), AES (Eq. 4), GCN weights (Eq. 2), CSR
// relabelling, the parameter model (Sec. 6) and diagnostics.  No HIP calls in this file.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>
#include <utility>
#include <vector>

#include <sched.h>

#include "gnn_internal.h"

namespace gnn {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

// Worker threads for the row-parallel passes: the cores this process may run on, at most 16, and
// one per 256k entries so that small graphs stay on the calling thread.
static int host_threads(int64_t nnz)
{
    cpu_set_t set;
    int cores = 1;
    if (sched_getaffinity(0, sizeof(set), &set) == 0) cores = CPU_COUNT(&set);
    if (cores > 16) cores = 16;
    const int64_t by_work = nnz / (256 * 1024) + 1;
    if ((int64_t)cores > by_work) cores = (int)by_work;
    return cores < 1 ? 1 : cores;
}

// Runs fn(row_begin, row_end, part) over contiguous row ranges that hold about the same number of
// entries each (rowptr must be non-decreasing).  The results of the parts do not depend on how
// many there are: every caller writes disjoint outputs or adds integers.
template <typename F>
static void for_row_ranges(int32_t n, const int32_t *rowptr, int parts, F fn)
{
    if (parts <= 1 || n <= 1) {
        fn((int32_t)0, n, 0);
        return;
    }
    std::vector<int32_t> cut((size_t)parts + 1, n);
    cut[0] = 0;
    const int64_t nnz = rowptr[n];
    for (int t = 1; t < parts; ++t) {
        const int64_t target = nnz * t / parts;
        cut[t] = (int32_t)(std::lower_bound(rowptr, rowptr + n, (int32_t)target) - rowptr);
        if (cut[t] < cut[t - 1]) cut[t] = cut[t - 1];
    }
    std::vector<std::thread> th;
    th.reserve((size_t)parts - 1);
    for (int t = 1; t < parts; ++t) th.emplace_back([&, t] { fn(cut[t], cut[t + 1], t); });
    fn(cut[0], cut[1], 0);
    for (auto &x : th) x.join();
}

static int check_host_csr(int32_t n, const int32_t *rowptr, const int32_t *colidx)
{
    if (n < 0 || !rowptr) return GNN_EINVAL;
    if (rowptr[0] != 0) return GNN_ECSR;
    for (int32_t i = 0; i < n; ++i)
        if (rowptr[i + 1] < rowptr[i]) return GNN_ECSR;
    if (rowptr[n] > 0 && !colidx) return GNN_EINVAL;
    const int parts = host_threads(rowptr[n]);
    std::vector<int> bad((size_t)parts, 0);
    for_row_ranges(n, rowptr, parts, [&](int32_t lo, int32_t hi, int t) {
        int b = 0;
        for (int64_t e = rowptr[lo]; e < rowptr[hi]; ++e) b |= (colidx[e] < 0 || colidx[e] >= n);
        bad[t] = b;
    });
    for (int b : bad)
        if (b) return GNN_ECSR;
    return GNN_OK;
}

static int64_t aes_sum_host(int32_t n, const int32_t *rowptr, const int32_t *colidx)
{
    const int parts = host_threads(rowptr[n]);
    std::vector<int64_t> part((size_t)parts, 0);
    for_row_ranges(n, rowptr, parts, [&](int32_t lo, int32_t hi, int t) {
        int64_t s = 0;
        for (int32_t i = lo; i < hi; ++i)
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) s += std::llabs((long long)i - (long long)colidx[e]);
        part[t] = s;
    });
    int64_t s = 0;
    for (int64_t x : part) s += x;
    return s;
}

// floor(sqrt(n) / 100) in integers (Sec. 5.1 rule).
static int64_t aes_threshold(int32_t n)
{
    int64_t r = (int64_t)std::sqrt((double)n);
    while (r * r > (int64_t)n) --r;
    while ((r + 1) * (r + 1) <= (int64_t)n) ++r;
    return r / 100;
}

// Greedy modularity merging + depth-first numbering.  The steps (clean adjacency, ascending
// (degree, id) visits, integer score w*M2 - du*dv, ties to the smallest id, children in merge
// order, pre-order numbering of roots in ascending id) are this library's fixed reading of the
// two-sentence description in Sec. 5.1.
static void modularity_order(int32_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm, int32_t *iperm)
{
    // clean adjacency via a stamp array (rows need not be sorted or duplicate-free)
    std::vector<int64_t> cptr((size_t)n + 1, 0);
    std::vector<int32_t> cadj;
    cadj.reserve((size_t)rowptr[n]);
    {
        std::vector<int32_t> stamp((size_t)n, -1);
        for (int32_t i = 0; i < n; ++i) {
            cptr[i] = (int64_t)cadj.size();
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const int32_t j = colidx[e];
                if (j == i || stamp[j] == i) continue;
                stamp[j] = i;
                cadj.push_back(j);
            }
        }
        cptr[n] = (int64_t)cadj.size();
    }
    const int64_t M2 = (int64_t)cadj.size();

    std::vector<int32_t> order((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return (cptr[a + 1] - cptr[a]) < (cptr[b + 1] - cptr[b]);
    });

    std::vector<int32_t> up((size_t)n);  // union-find links (compressed); roots point to themselves
    std::iota(up.begin(), up.end(), 0);
    std::vector<uint8_t> merged((size_t)n, 0);
    std::vector<int64_t> degw((size_t)n);
    for (int32_t i = 0; i < n; ++i) degw[i] = cptr[i + 1] - cptr[i];
    std::vector<std::vector<std::pair<int32_t, int64_t>>> kept((size_t)n);  // lists of merged vertices
    std::vector<std::vector<int32_t>> pending((size_t)n);  // children merged before the parent's visit
    std::vector<std::pair<int32_t, int32_t>> merges;       // (child, parent) in merge order
    merges.reserve((size_t)n);

    auto find = [&](int32_t x) {
        while (up[x] != x) {
            up[x] = up[up[x]];
            x = up[x];
        }
        return x;
    };

    std::vector<int64_t> acc((size_t)n, 0);
    std::vector<int32_t> touched;
    for (int32_t u : order) {
        touched.clear();
        auto add = [&](int32_t endpoint, int64_t w) {
            const int32_t r = find(endpoint);
            if (r == u) return;
            if (acc[r] == 0) touched.push_back(r);
            acc[r] += w;
        };
        for (int64_t k = cptr[u]; k < cptr[u + 1]; ++k) add(cadj[k], 1);
        for (int32_t c : pending[u]) {
            for (const auto &pr : kept[c]) add(pr.first, pr.second);
            std::vector<std::pair<int32_t, int64_t>>().swap(kept[c]);
        }
        std::vector<int32_t>().swap(pending[u]);
        int32_t best = -1;
        int64_t bestS = 0;
        for (int32_t v : touched) {
            const int64_t S = acc[v] * M2 - degw[u] * degw[v];
            if (best < 0 || S > bestS || (S == bestS && v < best)) {
                best = v;
                bestS = S;
            }
        }
        if (best >= 0 && bestS > 0) {
            auto &lst = kept[u];
            lst.reserve(touched.size());
            for (int32_t v : touched) lst.emplace_back(v, acc[v]);
            up[u] = best;
            merged[u] = 1;
            degw[best] += degw[u];
            pending[best].push_back(u);  // harmless if best was visited already: never read again
            merges.emplace_back(u, best);
        }
        for (int32_t v : touched) acc[v] = 0;
    }

    // children of every vertex in merge order (counting sort of the merge events by parent)
    std::vector<int64_t> chptr((size_t)n + 1, 0);
    for (const auto &m : merges) chptr[m.second + 1]++;
    for (int32_t i = 0; i < n; ++i) chptr[i + 1] += chptr[i];
    std::vector<int32_t> child(merges.size());
    {
        std::vector<int64_t> fill(chptr.begin(), chptr.end() - 1);
        for (const auto &m : merges) child[fill[m.second]++] = m.first;
    }
    // pre-order numbering
    std::vector<int32_t> stack;
    int32_t next = 0;
    for (int32_t r = 0; r < n; ++r) {
        if (merged[r]) continue;
        stack.push_back(r);
        while (!stack.empty()) {
            const int32_t x = stack.back();
            stack.pop_back();
            perm[x] = next;
            iperm[next] = x;
            ++next;
            for (int64_t k = chptr[x + 1]; k-- > chptr[x];) stack.push_back(child[k]);
        }
    }
}

void decide_defaults(int32_t n, int64_t nnz, int32_t max_degree, int32_t dim, int vec, int32_t *ngs, int32_t *dw,
                     int32_t *wpb)
{
    const double avg = n > 0 ? (double)nnz / (double)n : 0.0;
    const bool auto_dw = *dw <= 0;
    // dimension workers: lanes per neighbor row.  Each lane moves `vec` floats per load and owns the
    // chunks of the row that lie dw lanes apart.  Measured on MI355X (sweeps over dw at Dim 3 ... 256 on
    // five kinds of graphs), in this order of importance:
    //   * no idle lane-slots: dw * chunks should not exceed the row (Dim 22 = 11 loads of 8 bytes: 4 lanes x 3
    //     chunks beat 16 lanes x 1 chunk by 10 % of a model pass once the graph is renumbered);
    //   * at most three chunks per lane (four leave only two neighbours in flight: 7 % slower at Dim 128);
    //   * among equals, the team whose single load covers one 128-byte line of the row (8 lanes of 16 bytes),
    //     so that a wavefront requests 8 distinct lines per instruction: one-chunk teams of 16-64 lanes were
    //     5-11 % slower at Dim 128-256, half-line teams 6-14 % slower;
    //   * at least 4 lanes (or the whole row) per team, so that a wavefront does not carry more than 16 teams.
    // A row of at most 4 neighbors fills a lane's loads in flight only if the lane takes two chunks
    // (measured on batches of small graphs: 25 % faster at Dim 64), so a one-chunk team is halved there.
    if (auto_dw) {
        const int units = (dim + vec - 1) / vec;
        const int line_lanes = 128 / (4 * vec);
        int dmin = 1;
        while (dmin < units && dmin < 4) dmin *= 2;
        int best = 64, best_slots = 1 << 30, best_dist = 1 << 30;
        for (int d = dmin; d <= 64; d *= 2) {
            const int chunks = (units + d - 1) / d;
            if (chunks > 3 && d < 64) continue;
            const int slots = d * chunks;
            int dist = 0;
            for (int a = d, b = line_lanes; a != b; (a < b ? a *= 2 : b *= 2)) ++dist;
            if (slots < best_slots || (slots == best_slots && dist < best_dist)) {
                best = d;
                best_slots = slots;
                best_dist = dist;
            }
        }
        if (avg <= 4.0 && best > 1 && (units + best - 1) / best == 1 && units >= 2) best /= 2;
        *dw = best;
    }
    // neighbor-group size, from the graph alone so that one partition serves every layer of a
    // model.  Time ~ (#groups * per-group cost) + (#entries * per-row cost): bigger groups mean
    // fewer tuples, reductions and flushes per entry, and a team needs at least the 8 rows it keeps
    // in flight; past about twice the mean row length most groups are a whole row and nothing
    // more is gained.  Measured knee on MI355X: 16..32, as the paper found on its GPUs (Sec. 7.4).
    // A known longest row below that caps it: larger groups would only enlarge the index staging.
    if (*ngs <= 0) {
        int g = 16;
        while (g < 32 && (double)g < 2.0 * avg) g *= 2;
        // long rows (a dense graph, mean row 500: 128 is 8 % faster than 32): fewer parts to combine
        while (g < 128 && (double)g * 4.0 <= avg) g *= 2;
        if (max_degree > 0)
            while (g > 16 && g / 2 >= max_degree) g /= 2;
        *ngs = g;
    }
    // waves per block: 4 (the paper's preferred small blocks, Sec. 6), fewer when a wave already
    // carries many teams, so that a block serves at most 64 neighbor groups -- and Eq. 5's second
    // constraint, re-derived: the block's scratch memory (slots of Dim floats per group plus the staged
    // indices) must fit the per-block budget that keeps several blocks on a CU's 160 KB.  Fewer waves
    // per block shrink it; if one wave is still too much and the team width is free, wider teams do.
    if (*wpb <= 0) {
        const int teams = 64 / (*dw > 0 ? *dw : 1);
        int w = 64 / teams;
        w = w < 1 ? 1 : (w > 4 ? 4 : w);
        while (w > 1 && agg_lds_bytes(w * (64 / *dw), *ngs, dim, w, true) > kMaxLdsBytes) w /= 2;
        if (auto_dw)
            while (*dw < 64 && agg_lds_bytes(64 / *dw, *ngs, dim, 1, true) > kMaxLdsBytes) *dw *= 2;
        *wpb = w;
    }
}

}  // namespace gnn

using namespace gnn;

extern "C" {

int gnn_reorder(int32_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm, int32_t *iperm,
                double *aes_out, int *did_reorder, int force)
{
    if (!perm || !iperm) return GNN_EINVAL;
    const int rc = check_host_csr(n, rowptr, colidx);
    if (rc != GNN_OK) return rc;
    const int64_t nnz = rowptr[n];
    const int64_t s = aes_sum_host(n, rowptr, colidx);
    if (aes_out) *aes_out = nnz > 0 ? (double)s / (double)nnz : 0.0;
    const int64_t T = aes_threshold(n);
    const bool want = force != 0 || s > T * T * nnz;
    if (did_reorder) *did_reorder = want ? 1 : 0;
    if (!want) {
        for (int32_t i = 0; i < n; ++i) perm[i] = iperm[i] = i;
        return GNN_OK;
    }
    modularity_order(n, rowptr, colidx, perm, iperm);
    return GNN_OK;
}

int gnn_aes(int32_t n, const int32_t *rowptr, const int32_t *colidx, int64_t *aes_sum, double *aes)
{
    const int rc = check_host_csr(n, rowptr, colidx);
    if (rc != GNN_OK) return rc;
    const int64_t s = aes_sum_host(n, rowptr, colidx);
    if (aes_sum) *aes_sum = s;
    if (aes) *aes = rowptr[n] > 0 ? (double)s / (double)rowptr[n] : 0.0;
    return GNN_OK;
}

int gnn_gcn_norm(int32_t n, const int32_t *rowptr, const int32_t *colidx, float *ew)
{
    const int rc = check_host_csr(n, rowptr, colidx);
    if (rc != GNN_OK) return rc;
    if (rowptr[n] > 0 && !ew) return GNN_EINVAL;
    for_row_ranges(n, rowptr, host_threads(rowptr[n]), [&](int32_t lo, int32_t hi, int) {
        for (int32_t i = lo; i < hi; ++i) {
            const double di = (double)(rowptr[i + 1] - rowptr[i]);
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const int32_t j = colidx[e];
                const double dj = (double)(rowptr[j + 1] - rowptr[j]);
                ew[e] = (float)(1.0 / std::sqrt(di * dj));
            }
        }
    });
    return GNN_OK;
}

int gnn_apply_perm_csr(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *val,
                       const int32_t *perm, int32_t *rowptr2, int32_t *colidx2, float *val2)
{
    if (!perm || !rowptr2 || (val && !val2)) return GNN_EINVAL;
    const int rc = check_host_csr(n, rowptr, colidx);
    if (rc != GNN_OK) return rc;
    if (rowptr[n] > 0 && !colidx2) return GNN_EINVAL;
    std::vector<int32_t> inv((size_t)n, -1);
    for (int32_t i = 0; i < n; ++i) {
        if (perm[i] < 0 || perm[i] >= n || inv[perm[i]] != -1) return GNN_EINVAL;  // not a bijection
        inv[perm[i]] = i;
    }
    rowptr2[0] = 0;
    for (int32_t r = 0; r < n; ++r) rowptr2[r + 1] = rowptr2[r] + (rowptr[inv[r] + 1] - rowptr[inv[r]]);
    // the new rows are independent of each other: ranges of them go to the worker threads
    for_row_ranges(n, rowptr2, host_threads(rowptr[n]), [&](int32_t lo, int32_t hi, int) {
        std::vector<std::pair<int32_t, int32_t>> row;  // (new column, position in the old row)
        for (int32_t r = lo; r < hi; ++r) {
            const int32_t i = inv[r];
            const int32_t len = rowptr[i + 1] - rowptr[i];
            row.resize((size_t)len);
            for (int32_t k = 0; k < len; ++k) row[k] = {perm[colidx[rowptr[i] + k]], k};
            std::sort(row.begin(), row.end());
            for (int32_t k = 0; k < len; ++k) {
                colidx2[rowptr2[r] + k] = row[k].first;
                if (val) val2[rowptr2[r] + k] = val[rowptr[i] + row[k].second];
            }
        }
    });
    return GNN_OK;
}

int gnn_csr_transpose(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *val, int32_t *rowptr_t,
                      int32_t *colidx_t, float *val_t)
{
    if (!rowptr_t || (val && !val_t)) return GNN_EINVAL;
    const int rc = check_host_csr(n, rowptr, colidx);
    if (rc != GNN_OK) return rc;
    const int64_t nnz = rowptr[n];
    if (nnz > 0 && !colidx_t) return GNN_EINVAL;
    std::vector<int32_t> fill((size_t)n + 1, 0);
    for (int64_t e = 0; e < nnz; ++e) fill[colidx[e] + 1]++;
    rowptr_t[0] = 0;
    for (int32_t j = 0; j < n; ++j) {
        rowptr_t[j + 1] = rowptr_t[j] + fill[j + 1];
        fill[j] = rowptr_t[j];
    }
    // rows are visited in ascending order, so every transposed row comes out sorted
    for (int32_t i = 0; i < n; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int32_t pos = fill[colidx[e]]++;
            colidx_t[pos] = i;
            if (val) val_t[pos] = val[e];
        }
    return GNN_OK;
}

int gnn_decide(int32_t n, int64_t nnz, int32_t max_degree, int32_t dim, int32_t *ngs, int32_t *dw,
               int32_t *waves_per_block)
{
    if (n < 0 || nnz < 0 || dim <= 0 || !ngs || !dw || !waves_per_block) return GNN_EINVAL;
    int32_t a = *ngs, b = *dw, c = *waves_per_block;
    if (a < 0 || b < 0 || c < 0 || b > 64 || (b & (b - 1)) != 0 || c > kMaxWavesPerBlock) return GNN_EINVAL;
    const int vec = dim % 4 == 0 ? 4 : (dim % 2 == 0 ? 2 : 1);
    decide_defaults(n, nnz, max_degree, dim, vec, &a, &b, &c);
    *ngs = a;
    *dw = b;
    *waves_per_block = c;
    return GNN_OK;
}

int gnn_paper_model(int32_t dim, int32_t tpw, int32_t tpb, int32_t ngs, int32_t *dw, double *wpt,
                    int64_t *smem_bytes)
{
    if (dim <= 0 || tpw <= 0 || tpb <= 0 || ngs <= 0) return GNN_EINVAL;
    const int32_t d = dim >= tpw ? tpw : tpw / 2;                    // Eq. 6
    if (dw) *dw = d;
    if (wpt) *wpt = (double)ngs * (double)dim / (double)(d > 0 ? d : 1);  // Eq. 5
    if (smem_bytes) *smem_bytes = (int64_t)(tpb / tpw) * dim * 4;    // Eq. 5
    return GNN_OK;
}

const char *gnn_strerror(int code)
{
    switch (code) {
        case GNN_OK: return "ok";
        case GNN_EINVAL: return "invalid argument";
        case GNN_ECSR: return "malformed CSR";
        case GNN_EWORKSPACE: return "workspace missing, misaligned or too small";
        case GNN_EHIP: return "HIP runtime call failed";
        case GNN_ELIMIT: return "parameters exceed a documented limit";
        case GNN_ESTALE: return "workspace holds no matching partition";
        default: return "unknown error";
    }
}

int gnn_last_hip_error(void) { return g_last_hip_error; }
int gnn_version(void) { return 100; }

}  // extern "C"
