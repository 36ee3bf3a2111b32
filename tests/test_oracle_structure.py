"""Pins for the oracle's integer parts: neighbor partitioning, Algorithm 1, Eq. 4-6, renumbering."""
import numpy as np
import pytest

import oracle
from gnn_synth import config_graph
from util import csr_from_edges, random_sym_csr, read_golden


# ------------------------------------------------------------------ Sec. 4.1
def test_paper_worked_example_of_neighbor_groups():
    g = read_golden("ng_partition_example.txt")
    ngs = int(g["ngs"][0][0])
    rowptr = np.asarray(g["rowptr"][0], dtype=np.int32)
    node, start, end = oracle.ng_partition(rowptr, ngs)
    expect = np.asarray(g["ng"], dtype=np.int64)
    assert node.size == expect.shape[0] == 6
    assert np.array_equal(np.arange(6), expect[:, 0])
    assert np.array_equal(node, expect[:, 1])
    assert np.array_equal(start, expect[:, 2])
    assert np.array_equal(end, expect[:, 3])
    assert (node[2], start[2], end[2]) == (1, 4, 6)  # the tuple the paper prints for NG-2


@pytest.mark.parametrize("ngs", [1, 2, 3, 7, 32, 1000])
def test_neighbor_groups_tile_the_csr(ngs):
    rng = np.random.default_rng(ngs)
    deg = rng.integers(0, 40, size=200)
    deg[::17] = 0
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    node, start, end = oracle.ng_partition(rowptr, ngs)
    assert node.size == int(np.sum((deg + ngs - 1) // ngs))
    assert np.all(end > start) and np.all(end - start <= ngs)
    assert np.all(start >= rowptr[node]) and np.all(end <= rowptr[node + 1])  # never spans two rows
    if node.size:
        assert start[0] == rowptr[node[0]] and end[-1] == rowptr[-1]
        assert np.array_equal(start[1:], end[:-1])  # disjoint and gap-free in CSR order
    # only the last group of a row may be short
    short = (end - start) < ngs
    assert np.all(end[short] == rowptr[node[short] + 1])


# ------------------------------------------------------------------ Algorithm 1
def test_alg1_hand_trace():
    g = read_golden("alg1_trace.txt")
    nodes = np.asarray(g["nodes"][0], dtype=np.int32)
    slot, addr, leader = oracle.alg1_layout(nodes, int(g["warpPerBlock"][0][0]), int(g["dim"][0][0]))
    assert slot.tolist() == [int(x) for x in g["slot"][0]]
    assert leader.tolist() == [int(x) for x in g["leader"][0]]
    assert addr.tolist() == [int(x) for x in g["addr"][0]]


@pytest.mark.parametrize("wpb", [1, 2, 4, 16])
def test_alg1_invariants(wpb):
    rng = np.random.default_rng(wpb)
    nodes = np.sort(rng.integers(0, 60, size=333)).astype(np.int32)
    dim = 24
    slot, addr, leader = oracle.alg1_layout(nodes, wpb, dim)
    assert np.array_equal(addr, slot.astype(np.int64) * dim)
    for b0 in range(0, nodes.size, wpb):
        blk = slice(b0, min(b0 + wpb, nodes.size))
        nb, sb, lb = nodes[blk], slot[blk], leader[blk]
        assert lb[0] == 1 and sb[0] == 0  # first worker of a block: leader, slot 0
        assert sb.max() < wpb
        assert sb.max() + 1 == len(np.unique(nb))  # one slot per distinct target node
        for k in range(1, len(nb)):
            if nb[k] == nb[k - 1]:
                assert sb[k] == sb[k - 1] and lb[k] == 0
            else:
                assert sb[k] == sb[k - 1] + 1 and lb[k] == 1
    # leaders = distinct (block, node) pairs: the number of row flushes to global memory
    pairs = {(i // wpb, int(v)) for i, v in enumerate(nodes)}
    assert int(leader.sum()) == len(pairs)


# ------------------------------------------------------------------ Eq. 5 / Eq. 6 as printed
def test_eq5_eq6_literal_values():
    assert oracle.eq6_dw(16, 32) == 16
    assert oracle.eq6_dw(64, 32) == 32
    assert oracle.eq6_dw(32, 32) == 32
    assert oracle.eq5_smem(128, 32, 64) == 1024
    assert oracle.eq5_wpt(32, 64, 32) == 64.0
    assert oracle.eq5_wpt(3, 16, 16) == 3.0


# ------------------------------------------------------------------ Eq. 4
def test_aes_hand_computed():
    # path 0-1-2-3: stored entries (0,1)(1,0)(1,2)(2,1)(2,3)(3,2) -> spans all 1
    rp, ci = csr_from_edges(4, [(0, 1), (1, 2), (2, 3)])
    assert oracle.aes_sum(rp, ci) == 6 and oracle.aes(rp, ci) == 1.0
    # edges 0-3, 1-2: spans 3,3,1,1 -> 8/4
    rp, ci = csr_from_edges(4, [(0, 3), (1, 2)])
    assert oracle.aes_sum(rp, ci) == 8 and oracle.aes(rp, ci) == 2.0
    # self loops add entries of span 0
    rp, ci = csr_from_edges(4, [(0, 3), (1, 2)], self_loops=True)
    assert oracle.aes_sum(rp, ci) == 8 and oracle.aes(rp, ci) == 1.0


def test_aes_thresholds_from_the_rule():
    assert oracle.aes_threshold(2708) == 0
    assert oracle.aes_threshold(9999) == 0
    assert oracle.aes_threshold(10000) == 1
    assert oracle.aes_threshold(410236) == 6
    assert oracle.aes_threshold(1 << 20) == 10
    # rule: sqrt(AES) > T.  A path graph of 40,000 nodes has AES = 1, T = 2 -> no reordering
    n = 40000
    rp, ci = csr_from_edges(n, [(i, i + 1) for i in range(n - 1)])
    assert oracle.aes_sum(rp, ci) == 2 * (n - 1)
    assert not oracle.should_reorder(rp, ci)
    # the same count of edges with span 5: AES = 5 > 4 = T^2 -> reorder
    rp2, ci2 = csr_from_edges(n, [(i, i + 5) for i in range(0, n - 5)])
    assert oracle.should_reorder(rp2, ci2)
    # small graphs (T = 0): any non-loop edge triggers it
    rp3, ci3 = csr_from_edges(5, [(0, 1)])
    assert oracle.should_reorder(rp3, ci3)
    assert not oracle.should_reorder(*csr_from_edges(5, [], self_loops=True))


# ------------------------------------------------------------------ Sec. 5.1 renumbering
def _modularity(rp, ci, label):
    n = len(rp) - 1
    rows = np.repeat(np.arange(n), np.diff(rp))
    keep = rows != ci
    rows, cols = rows[keep], ci[keep]
    m2 = rows.size
    deg = np.bincount(rows, minlength=n).astype(np.float64)
    inside = np.sum(label[rows] == label[cols]) / m2
    tot = np.bincount(label, weights=deg)
    return inside - np.sum((tot / m2) ** 2)


def test_reorder_hand_trace():
    g = read_golden("reorder_trace.txt")
    n = int(g["n"][0][0])
    edges = [tuple(int(x) for x in t.split("-")) for t in g["edges"][0]]
    rp, ci = csr_from_edges(n, edges)
    perm, iperm = oracle.reorder(rp, ci)
    assert perm.tolist() == [int(x) for x in g["perm"][0]]
    assert iperm.tolist() == [int(x) for x in g["iperm"][0]]
    # self loops and duplicate entries do not change the result
    rp2, ci2 = csr_from_edges(n, edges, self_loops=True)
    assert oracle.reorder(rp2, ci2)[0].tolist() == perm.tolist()


def test_reorder_is_a_bijection_and_deterministic():
    g = config_graph(2, shrink=8)
    p1, ip1 = oracle.reorder(g.rowptr, g.colidx)
    p2, ip2 = oracle.reorder(g.rowptr.copy(), g.colidx.copy())
    assert np.array_equal(p1, p2) and np.array_equal(ip1, ip2)
    assert np.array_equal(np.sort(p1), np.arange(g.n))
    assert np.array_equal(ip1[p1], np.arange(g.n))


def test_reorder_makes_interleaved_cliques_contiguous():
    k = 6
    a = [2 * i for i in range(k)]
    b = [2 * i + 1 for i in range(k)]
    edges = [(x, y) for s in (a, b) for x in s for y in s if x < y]
    rp, ci = csr_from_edges(2 * k, edges)
    perm, _ = oracle.reorder(rp, ci)
    for s in (a, b):
        ids = np.sort(perm[s])
        assert ids[-1] - ids[0] == k - 1


def test_reorder_lowers_aes_of_shuffled_block_diagonal_batch():
    g = config_graph(3, shrink=8)
    rng = np.random.default_rng(0)
    label = rng.permutation(g.n).astype(np.int32)
    rp_s, ci_s = oracle.apply_perm_csr(g.rowptr, g.colidx, label)
    aes_shuffled = oracle.aes(rp_s, ci_s)
    perm, _ = oracle.reorder(rp_s, ci_s)
    rp_r, ci_r = oracle.apply_perm_csr(rp_s, ci_s, perm)
    aes_after = oracle.aes(rp_r, ci_r)
    assert aes_after < 0.02 * aes_shuffled
    assert aes_after < 4 * oracle.aes(g.rowptr, g.colidx)
    # every small graph is a connected component: after renumbering each one is a contiguous id range
    sizes = g.meta.get("graph_sizes")
    if sizes is not None:
        off = np.concatenate([[0], np.cumsum(sizes)])
        new = perm[label]
        for k in range(len(sizes)):
            ids = new[off[k]:off[k + 1]]
            assert ids.max() - ids.min() == len(ids) - 1


def test_reorder_finds_planted_communities():
    g = config_graph(4, shrink=64, variant="shuffled")
    perm, _ = oracle.reorder(g.rowptr, g.colidx)
    rp_r, ci_r = oracle.apply_perm_csr(g.rowptr, g.colidx, perm)
    assert oracle.aes(rp_r, ci_r) < 0.5 * oracle.aes(g.rowptr, g.colidx)
    # contiguous chunks of the new numbering form a clustering with clearly positive modularity,
    # which random labels (the shuffled ids) do not
    chunk = 256
    q_new = _modularity(g.rowptr, g.colidx, (perm // chunk).astype(np.int64))
    q_old = _modularity(g.rowptr, g.colidx, (np.arange(g.n) // chunk).astype(np.int64))
    assert q_new > 0.3 and q_old < 0.05


def test_reorder_path_graph_keeps_small_span():
    n = 500
    rp, ci = csr_from_edges(n, [(i, i + 1) for i in range(n - 1)])
    perm, _ = oracle.reorder(rp, ci)
    rp_r, ci_r = oracle.apply_perm_csr(rp, ci, perm)
    assert oracle.aes(rp_r, ci_r) < 8.0


def test_apply_perm_csr_and_permute_rows():
    rng = np.random.default_rng(4)
    n = 40
    rp, ci = random_sym_csr(n, 0.15, rng, self_loops=True)
    val = rng.standard_normal(ci.size).astype(np.float32)
    perm = rng.permutation(n).astype(np.int32)
    rp2, ci2, v2 = oracle.apply_perm_csr(rp, ci, perm, val)
    A = {(i, int(ci[e])): val[e] for i in range(n) for e in range(rp[i], rp[i + 1])}
    B = {(i, int(ci2[e])): v2[e] for i in range(n) for e in range(rp2[i], rp2[i + 1])}
    assert B == {(int(perm[i]), int(perm[j])): v for (i, j), v in A.items()}
    for i in range(n):
        assert np.all(np.diff(ci2[rp2[i]:rp2[i + 1]]) > 0)
    X = rng.standard_normal((n, 5)).astype(np.float32)
    Y = oracle.permute_rows(X, perm)
    assert np.array_equal(Y[perm], X)
    iperm = np.argsort(perm).astype(np.int32)
    assert np.array_equal(oracle.permute_rows(Y, iperm), X)


@pytest.mark.parametrize("kind", ["gcn", "gin"])
def test_renumbering_leaves_the_aggregation_unchanged(kind):
    # P(A X) = (P A P^T)(P X); with integer-valued data every sum is exact -> bitwise equality
    rng = np.random.default_rng(8)
    g = config_graph(1, shrink=4)
    perm, iperm = oracle.reorder(g.rowptr, g.colidx)
    X = rng.integers(-4, 5, size=(g.n, 8)).astype(np.float32)
    Xp = oracle.permute_rows(X, perm)
    if kind == "gin":
        base = oracle.aggregate_gin(g.rowptr, g.colidx, 1.0, X)
        rp2, ci2 = oracle.apply_perm_csr(g.rowptr, g.colidx, perm)
        moved = oracle.aggregate_gin(rp2, ci2, 1.0, Xp)
    else:
        w = rng.integers(1, 5, size=g.nnz).astype(np.float32)
        base = oracle.aggregate_gcn(g.rowptr, g.colidx, w, X)
        rp2, ci2, w2 = oracle.apply_perm_csr(g.rowptr, g.colidx, perm, w)
        moved = oracle.aggregate_gcn(rp2, ci2, w2, Xp)
    assert np.array_equal(oracle.permute_rows(moved, iperm), base)
    # and with the real normalisation weights, to rounding
    if kind == "gcn":
        ew = oracle.gcn_norm(g.rowptr, g.colidx)
        Xf = rng.standard_normal((g.n, 8)).astype(np.float32)
        base = oracle.aggregate_gcn(g.rowptr, g.colidx, ew, Xf)
        rp2, ci2 = oracle.apply_perm_csr(g.rowptr, g.colidx, perm)
        moved = oracle.aggregate_gcn(rp2, ci2, oracle.gcn_norm(rp2, ci2), oracle.permute_rows(Xf, perm))
        np.testing.assert_allclose(oracle.permute_rows(moved, iperm), base, rtol=0, atol=1e-6)


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (4, 32), (5, 64)])
@pytest.mark.parametrize("ngs,T", [(2, 4), (4, 16), (16, 16), (32, 64)])
def test_global_flushes_per_block_are_bounded(cfg, shrink, ngs, T):
    # Sec. 5.2: a node whose groups span blocks costs one global flush of Dim values per (node, block),
    # however many groups (k * ngs neighbours) of it the block holds.  With groups in CSR order only the
    # node of a block's first group and the node of its last group can continue outside the block, so a
    # block flushes at most two partial rows -- what the atomic count of the ablation study measures
    # and what the two scratch rows per block of the ordered flush rely on.
    g = config_graph(cfg, shrink=shrink)
    node, start, end = oracle.ng_partition(g.rowptr, ngs)
    slot, _, leader = oracle.alg1_layout(node, T, 1)
    groups_of = np.bincount(node, minlength=g.n)
    first_group = np.concatenate([[0], np.cumsum(groups_of)[:-1]])
    flushes, pairs = 0, 0
    for b0 in range(0, node.size, T):
        blk = node[b0:b0 + T]
        leaders = np.flatnonzero(leader[b0:b0 + T])
        assert leaders.size == np.unique(blk).size          # one leader per (block, node) pair
        pairs += leaders.size
        partial = []
        for l in leaders:
            v = blk[l]
            inside = first_group[v] >= b0 and first_group[v] + groups_of[v] <= b0 + blk.size
            if not inside:
                partial.append(int(l))
        assert len(partial) <= 2
        for l in partial:                                   # only the block's first or last node
            assert blk[l] == blk[0] or blk[l] == blk[-1]
        flushes += len(partial)
    blocks = (node.size + T - 1) // T
    assert flushes <= 2 * blocks
    # without block-level accumulation every group would flush: the paper's reduction of atomics
    assert flushes <= node.size and pairs <= node.size
