"""Pins of the oracle's aggregation with a feature vector on every stored entry (Sec. 3.1 of the paper: the
second class of aggregation applies edge features to each neighbor).  The reading taken here:
out[i, :] = sum over stored entries e = (i, j) of E[e, :] * X[j, :], elementwise.  Every test below compares
the oracle with something it does not contain: a dense tensor expression written with numpy, the scalar-weight
aggregation (pinned elsewhere) that it must reduce to, values worked by hand."""
import numpy as np
import pytest

import oracle
from gnn_synth import config_graph


def _random_csr(n, p, seed):
    rng = np.random.default_rng(seed)
    A = rng.random((n, n)) < p
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(A.sum(1))
    colidx = np.nonzero(A)[1].astype(np.int32)
    return A, rowptr, colidx


@pytest.mark.parametrize("n,dim,p", [(7, 3, 0.5), (23, 16, 0.2), (40, 5, 0.1)])
def test_matches_the_dense_tensor_expression(n, dim, p):
    A, rowptr, colidx = _random_csr(n, p, seed=n + dim)
    rng = np.random.default_rng(dim)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    E = rng.standard_normal((colidx.size, dim)).astype(np.float32)
    # dense tensor T[i, j, :] = feature vector of entry (i, j), zero where there is no entry
    T = np.zeros((n, n, dim))
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    T[rows, colidx, :] = E
    want = np.einsum("ijk,jk->ik", T, X.astype(np.float64))
    got, ab = oracle.aggregate_edge_vec(rowptr, colidx, E, X, want_abs=True)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(ab, np.einsum("ijk,jk->ik", np.abs(T), np.abs(X.astype(np.float64))), rtol=1e-12)
    # not symmetric in its operands: the vector belongs to the entry, the row to the entry's column
    assert not np.allclose(got, np.einsum("ijk,ik->ik", T, X.astype(np.float64)), atol=1e-3)


def test_constant_vectors_reduce_to_the_weighted_sum():
    g = config_graph(4, shrink=64)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((g.n, 12)).astype(np.float32)
    w = rng.standard_normal(g.nnz).astype(np.float32)
    E = np.repeat(w[:, None], 12, axis=1)
    got = oracle.aggregate_edge_vec(g.rowptr, g.colidx, E, X)
    want = oracle.aggregate_gcn(g.rowptr, g.colidx, w, X)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    ones = np.ones((g.nnz, 12), dtype=np.float32)
    assert np.array_equal(oracle.aggregate_edge_vec(g.rowptr, g.colidx, ones, X), oracle.aggregate_gcn(g.rowptr, g.colidx, None, X))


def test_one_hot_vectors_select_single_dimensions():
    # entry e keeps only dimension e mod dim of its neighbour row: a transposed or shifted index shows at once
    A, rowptr, colidx = _random_csr(15, 0.3, seed=3)
    dim = 4
    X = np.arange(15 * dim, dtype=np.float32).reshape(15, dim) + 1
    E = np.zeros((colidx.size, dim), dtype=np.float32)
    E[np.arange(colidx.size), np.arange(colidx.size) % dim] = 1.0
    got = oracle.aggregate_edge_vec(rowptr, colidx, E, X)
    want = np.zeros((15, dim))
    for i in range(15):
        for e in range(rowptr[i], rowptr[i + 1]):
            want[i, e % dim] += X[colidx[e], e % dim]
    assert np.array_equal(got, want.astype(np.float32))


def test_hand_worked_triangle():
    # nodes 0, 1, 2; entries in CSR order: (0,1) (0,2) (1,0) (2,0) (2,1); two dimensions
    rowptr = np.array([0, 2, 3, 5], dtype=np.int32)
    colidx = np.array([1, 2, 0, 0, 1], dtype=np.int32)
    X = np.array([[1, 10], [2, 20], [3, 30]], dtype=np.float32)
    E = np.array([[1, 0], [2, 1], [-1, 1], [0.5, 0.5], [0, -2]], dtype=np.float32)
    got = oracle.aggregate_edge_vec(rowptr, colidx, E, X)
    # row 0: 1*[2,20]*[1,0] + [3,30]*[2,1] = [2+6, 0+30]; row 1: [1,10]*[-1,1]; row 2: [1,10]*[.5,.5] + [2,20]*[0,-2]
    assert np.array_equal(got, np.array([[8, 30], [-1, 10], [0.5, 5 - 40]], dtype=np.float32))
    # a node without entries and an empty graph
    assert np.array_equal(oracle.aggregate_edge_vec(np.array([0, 0, 1], dtype=np.int32), np.array([0], dtype=np.int32),
                                                    np.array([[2, 3]], dtype=np.float32), X[:2]), np.array([[0, 0], [2, 30]], dtype=np.float32))


def test_renumbering_invariance():
    g = config_graph(3, shrink=16)
    rng = np.random.default_rng(9)
    dim = 6
    X = rng.integers(-3, 4, size=(g.n, dim)).astype(np.float32)
    E = rng.integers(-2, 3, size=(g.nnz, dim)).astype(np.float32)
    ref = oracle.aggregate_edge_vec(g.rowptr, g.colidx, E, X)
    perm = rng.permutation(g.n).astype(np.int32)  # perm[old] = new
    # relabel by hand: new row perm[i] holds the entries of old row i with columns perm[j], vectors moving along
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    order = np.lexsort((perm[g.colidx], perm[rows]))
    new_rows = perm[rows][order]
    rp2 = np.zeros(g.n + 1, dtype=np.int32)
    rp2[1:] = np.cumsum(np.bincount(new_rows, minlength=g.n))
    ci2 = perm[g.colidx][order].astype(np.int32)
    E2 = E[order]
    X2 = np.empty_like(X)
    X2[perm] = X
    got = oracle.aggregate_edge_vec(rp2, ci2, E2, X2)
    assert np.array_equal(got[perm], ref)  # integer data: exact in any order
