"""Pins for the oracle's aggregation, normalisation and dense layer (CPU only)."""
import numpy as np
import pytest

import oracle
from util import csr_from_edges, dense_from_csr, random_sym_csr


@pytest.mark.parametrize("n,p,dim,seed", [(1, 0.0, 3, 0), (7, 0.5, 5, 1), (33, 0.2, 16, 2), (64, 0.1, 7, 3)])
def test_gcn_matches_dense_product(n, p, dim, seed):
    rng = np.random.default_rng(seed)
    rp, ci = random_sym_csr(n, p, rng, self_loops=True)
    ew = rng.standard_normal(ci.size).astype(np.float32)  # arbitrary weights: pins the pairing of ew with colidx
    X = rng.standard_normal((n, dim)).astype(np.float32)
    ref = dense_from_csr(rp, ci, ew) @ X.astype(np.float64)
    out, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-6 * max(1.0, np.abs(ref).max()))
    assert np.array_equal(out, ref.astype(np.float32))  # double accumulate, one rounding
    ref_abs = np.abs(dense_from_csr(rp, ci, np.abs(ew))) @ np.abs(X.astype(np.float64))
    np.testing.assert_allclose(ab, ref_abs, rtol=1e-12)


def test_gcn_is_not_symmetric_in_its_operands():
    # a directed (non-symmetric) pattern catches a transposed operand
    rp = np.array([0, 2, 2, 3], dtype=np.int32)
    ci = np.array([1, 2, 0], dtype=np.int32)
    ew = np.array([2.0, 3.0, 5.0], dtype=np.float32)
    X = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]], dtype=np.float32)
    out = oracle.aggregate_gcn(rp, ci, ew, X)
    assert out.tolist() == [[2 * 2 + 3 * 4, 2 * 20 + 3 * 40], [0, 0], [5, 50]]


@pytest.mark.parametrize("n,p,dim,eps,seed", [(1, 0, 2, 0.0, 0), (9, 0.4, 4, 0.0, 1), (40, 0.15, 64, 0.25, 2)])
def test_gin_matches_dense_product(n, p, dim, eps, seed):
    rng = np.random.default_rng(seed)
    rp, ci = random_sym_csr(n, p, rng)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    A = dense_from_csr(rp, ci) + (1.0 + float(np.float32(eps))) * np.eye(n)
    ref = A @ X.astype(np.float64)
    out = oracle.aggregate_gin(rp, ci, eps, X)
    assert np.array_equal(out, ref.astype(np.float32))


def test_all_ones_features_give_normalised_degree_sums():
    rng = np.random.default_rng(5)
    n = 50
    rp, ci = random_sym_csr(n, 0.1, rng, self_loops=True)
    ew = oracle.gcn_norm(rp, ci)
    d = np.diff(rp).astype(np.float64)
    out = oracle.aggregate_gcn(rp, ci, ew, np.ones((n, 3), dtype=np.float32))
    for i in range(n):
        expect = sum(float(np.float32(1.0 / np.sqrt(d[i] * d[j]))) for j in ci[rp[i]:rp[i + 1]])
        assert out[i, 0] == np.float32(expect)
        assert out[i, 0] == out[i, 1] == out[i, 2]
    gin = oracle.aggregate_gin(rp, ci, 0.5, np.ones((n, 2), dtype=np.float32))
    assert np.array_equal(gin[:, 0], (1.5 + d).astype(np.float32))


@pytest.mark.parametrize("n,k", [(8, 2), (12, 4), (9, 8)])
def test_regular_graph_with_self_loops_aggregates_ones_to_one(n, k):
    # circulant graph: i ~ i +- 1..k/2  -> k-regular; with self loops every weight is 1/(k+1)
    edges = [(i, (i + s) % n) for i in range(n) for s in range(1, k // 2 + 1)]
    rp, ci = csr_from_edges(n, edges, self_loops=True)
    assert np.all(np.diff(rp) == k + 1)
    ew = oracle.gcn_norm(rp, ci)
    assert np.all(ew == np.float32(1.0 / (k + 1)))
    out = oracle.aggregate_gcn(rp, ci, ew, np.ones((n, 4), dtype=np.float32))
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=2e-7)


def test_star_graph_closed_form():
    n = 17  # centre 0 plus 16 leaves, self loops on
    rp, ci = csr_from_edges(n, [(0, i) for i in range(1, n)], self_loops=True)
    ew = oracle.gcn_norm(rp, ci)
    out = oracle.aggregate_gcn(rp, ci, ew, np.ones((n, 1), dtype=np.float32))
    centre = 1.0 / n + (n - 1) / np.sqrt(2.0 * n)
    leaf = 0.5 + 1.0 / np.sqrt(2.0 * n)
    assert abs(out[0, 0] - centre) < 1e-6
    np.testing.assert_allclose(out[1:, 0], leaf, rtol=0, atol=1e-6)


def test_gcn_norm_is_symmetric_bitwise():
    rng = np.random.default_rng(11)
    rp, ci = random_sym_csr(60, 0.1, rng, self_loops=True)
    ew = oracle.gcn_norm(rp, ci)
    pos = {(i, int(ci[e])): e for i in range(60) for e in range(rp[i], rp[i + 1])}
    for (i, j), e in pos.items():
        assert ew[e] == ew[pos[(j, i)]]
    d = np.diff(rp)
    e = pos[(3, 3)]
    assert ew[e] == np.float32(1.0 / d[3])


def test_linearity_and_eps_term():
    rng = np.random.default_rng(7)
    n, dim = 30, 6
    rp, ci = random_sym_csr(n, 0.2, rng)
    # integer-valued inputs: every sum is exact, so linear identities hold bitwise
    X = rng.integers(-8, 9, size=(n, dim)).astype(np.float32)
    Y = rng.integers(-8, 9, size=(n, dim)).astype(np.float32)
    a0 = oracle.aggregate_gin(rp, ci, 0.0, X)
    assert np.array_equal(oracle.aggregate_gin(rp, ci, 0.0, X + Y), a0 + oracle.aggregate_gin(rp, ci, 0.0, Y))
    assert np.array_equal(oracle.aggregate_gin(rp, ci, 0.5, X) - a0, 0.5 * X)
    ew = rng.integers(1, 4, size=ci.size).astype(np.float32)
    g = oracle.aggregate_gcn(rp, ci, ew, X)
    assert np.array_equal(oracle.aggregate_gcn(rp, ci, ew, 2 * X + Y), 2 * g + oracle.aggregate_gcn(rp, ci, ew, Y))
    assert np.array_equal(oracle.aggregate_gcn(rp, ci, None, X), a0 - X)  # unit weights = plain neighbour sum


def test_empty_graph_and_isolated_nodes():
    X = np.arange(12, dtype=np.float32).reshape(4, 3)
    rp = np.zeros(5, dtype=np.int32)
    ci = np.zeros(0, dtype=np.int32)
    assert np.array_equal(oracle.aggregate_gcn(rp, ci, np.zeros(0, np.float32), X), np.zeros((4, 3), np.float32))
    assert np.array_equal(oracle.aggregate_gin(rp, ci, 1.0, X), 2 * X)


@pytest.mark.parametrize("n,K,M,relu,bias", [(5, 1, 3, False, False), (17, 9, 4, True, True), (33, 64, 64, True, False)])
def test_gemm_matches_numpy(n, K, M, relu, bias):
    rng = np.random.default_rng(n)
    A = rng.standard_normal((n, K)).astype(np.float32)
    W = rng.standard_normal((K, M)).astype(np.float32)
    b = rng.standard_normal(M).astype(np.float32) if bias else None
    ref = A.astype(np.float64) @ W.astype(np.float64)
    if bias:
        ref = ref + b.astype(np.float64)
    if relu:
        ref = np.maximum(ref, 0.0)
    out = oracle.gemm_bias_act(A, W, b, relu)
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-6)


def test_gemm_identity_and_non_square_orientation():
    A = np.arange(12, dtype=np.float32).reshape(3, 4)
    assert np.array_equal(oracle.gemm_bias_act(A, np.eye(4, dtype=np.float32)), A)
    W = np.zeros((4, 2), dtype=np.float32)
    W[1, 0] = 1.0
    W[3, 1] = 2.0
    assert np.array_equal(oracle.gemm_bias_act(A, W), np.stack([A[:, 1], 2 * A[:, 3]], axis=1))


def test_layer_order_gcn_update_first_gin_aggregate_first():
    rng = np.random.default_rng(3)
    n = 20
    rp, ci = random_sym_csr(n, 0.3, rng, self_loops=True)
    ew = oracle.gcn_norm(rp, ci)
    X = rng.standard_normal((n, 8)).astype(np.float32)
    W = rng.standard_normal((8, 3)).astype(np.float32)
    A = dense_from_csr(rp, ci, ew)
    ref = np.maximum(A @ (X.astype(np.float64) @ W.astype(np.float64)), 0)
    np.testing.assert_allclose(oracle.gcn_layer(rp, ci, ew, X, W, None, True), ref, rtol=1e-5, atol=1e-6)
    rp2, ci2 = random_sym_csr(n, 0.3, rng)
    G = dense_from_csr(rp2, ci2) + np.eye(n)
    b = rng.standard_normal(3).astype(np.float32)
    ref2 = np.maximum((G @ X.astype(np.float64)) @ W.astype(np.float64) + b, 0)
    np.testing.assert_allclose(oracle.gin_layer(rp2, ci2, 0.0, X, W, b, True), ref2, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("cfg,shrink,dim", [(2, 1, 16), (4, 32, 24), (5, 64, 7)])
def test_oracle_against_a_library_sparse_product(cfg, shrink, dim):
    """The aggregation is a sparse x dense product: scipy's CSR product in fp64 on graphs of a few
    thousand to tens of thousands of nodes (brute force covers only tiny ones), GCN weights, GIN self
    term, and the max / min / mean reductions through scipy's own row operations."""
    import scipy.sparse as sp
    from gnn_synth import config_graph, features
    g = config_graph(cfg, shrink=shrink)
    n = g.n
    X = features(n, dim, seed=cfg * 10 + dim)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    A = sp.csr_matrix((ew.astype(np.float64), g.colidx, g.rowptr), shape=(n, n))
    ref = (A @ X.astype(np.float64)).astype(np.float32)
    got = oracle.aggregate_gcn(g.rowptr, g.colidx, ew, X)
    assert np.abs(got - ref).max() <= 2e-7 * max(1.0, np.abs(ref).max())
    ones = sp.csr_matrix((np.ones(g.nnz), g.colidx, g.rowptr), shape=(n, n))
    eps = 0.25
    ref = ((1.0 + eps) * X.astype(np.float64) + ones @ X.astype(np.float64)).astype(np.float32)
    got = oracle.aggregate_gin(g.rowptr, g.colidx, eps, X)
    assert np.abs(got - ref).max() <= 2e-7 * max(1.0, np.abs(ref).max())
    deg = np.diff(g.rowptr).astype(np.float64)
    mean = np.divide((ones @ X.astype(np.float64)), deg[:, None], out=np.zeros((n, dim)), where=deg[:, None] > 0)
    got = oracle.aggregate_reduce(g.rowptr, g.colidx, X, oracle.REDUCE_MEAN)
    assert np.abs(got - mean.astype(np.float32)).max() <= 2e-7 * max(1.0, np.abs(mean).max())
    # max over the stored entries of a row: numpy's reduceat over the gathered rows (rows without entries give 0)
    nonempty = np.flatnonzero(deg > 0)
    gathered = X[g.colidx]
    mx = np.zeros((n, dim), dtype=np.float32)
    mx[nonempty] = np.maximum.reduceat(gathered, g.rowptr[:-1][nonempty].astype(np.int64), axis=0)
    assert np.array_equal(oracle.aggregate_reduce(g.rowptr, g.colidx, X, oracle.REDUCE_MAX), mx)
