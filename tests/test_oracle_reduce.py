"""Pins for the oracle's max / min / mean aggregation (Sec. 3.1: aggregation over neighbour
embeddings only), CPU only: numpy reductions over explicit neighbour lists, closed forms, order
relations and the link to the sum aggregation."""
import numpy as np
import pytest

import oracle
from util import csr_from_edges, random_sym_csr

MAX, MIN, MEAN = oracle.REDUCE_MAX, oracle.REDUCE_MIN, oracle.REDUCE_MEAN


def _directed(n, avg, rng):
    deg = rng.integers(0, 2 * avg + 1, size=n)
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    ci = rng.integers(0, n, size=int(rp[-1])).astype(np.int32)  # duplicates and self entries allowed
    return rp, ci


@pytest.mark.parametrize("n,dim,seed", [(1, 3, 0), (9, 4, 1), (40, 17, 2), (64, 64, 3)])
def test_reductions_match_numpy_over_explicit_neighbour_lists(n, dim, seed):
    rng = np.random.default_rng(seed)
    rp, ci = _directed(n, 3, rng)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    got = {op: oracle.aggregate_reduce(rp, ci, X, op) for op in (MAX, MIN, MEAN)}
    for i in range(n):
        nb = ci[rp[i]:rp[i + 1]]
        if nb.size == 0:
            for op in (MAX, MIN, MEAN):
                assert not got[op][i].any()  # nothing to reduce: zero row
            continue
        rows = X[nb]
        assert np.array_equal(got[MAX][i], rows.max(axis=0))  # comparisons do not round: exact
        assert np.array_equal(got[MIN][i], rows.min(axis=0))
        assert np.array_equal(got[MEAN][i], (rows.astype(np.float64).sum(axis=0) / nb.size).astype(np.float32))


def test_closed_forms_on_a_path_and_a_star():
    # path 0-1-2-3-4 with feature = node id: max is the larger neighbour, min the smaller
    rp, ci = csr_from_edges(5, [(i, i + 1) for i in range(4)])
    X = np.arange(5, dtype=np.float32)[:, None] * np.array([[1.0, -1.0]], dtype=np.float32)
    mx, mn, me = (oracle.aggregate_reduce(rp, ci, X, op) for op in (MAX, MIN, MEAN))
    assert mx[:, 0].tolist() == [1, 2, 3, 4, 3] and mn[:, 0].tolist() == [1, 0, 1, 2, 3]
    assert mx[:, 1].tolist() == [-1, 0, -1, -2, -3] and mn[:, 1].tolist() == [-1, -2, -3, -4, -3]  # sign flips swap them
    assert me[:, 0].tolist() == [1, 1, 2, 3, 3]
    # star with centre 0 and 6 leaves: the centre sees all leaves, a leaf sees only the centre
    rp, ci = csr_from_edges(7, [(0, i) for i in range(1, 7)])
    X = np.array([[10.0], [1.0], [2.0], [3.0], [4.0], [5.0], [6.0]], dtype=np.float32)
    assert oracle.aggregate_reduce(rp, ci, X, MAX)[:, 0].tolist() == [6, 10, 10, 10, 10, 10, 10]
    assert oracle.aggregate_reduce(rp, ci, X, MIN)[:, 0].tolist() == [1, 10, 10, 10, 10, 10, 10]
    assert oracle.aggregate_reduce(rp, ci, X, MEAN)[:, 0].tolist() == [3.5, 10, 10, 10, 10, 10, 10]


def test_order_relations_and_link_to_the_sum_aggregation():
    rng = np.random.default_rng(5)
    rp, ci = random_sym_csr(80, 0.08, rng)
    X = rng.standard_normal((80, 12)).astype(np.float32)
    mx, mn = oracle.aggregate_reduce(rp, ci, X, MAX), oracle.aggregate_reduce(rp, ci, X, MIN)
    me, ab = oracle.aggregate_reduce(rp, ci, X, MEAN, want_abs=True)
    deg = np.diff(rp)[:, None]
    has = (deg > 0).repeat(12, axis=1)
    assert (mn[has] <= me[has] + 1e-6).all() and (me[has] <= mx[has] + 1e-6).all()
    # mean * degree equals the unweighted sum aggregation (Eq. 2 with unit weights) up to one rounding
    s = oracle.aggregate_gcn(rp, ci, None, X).astype(np.float64)
    np.testing.assert_allclose(me.astype(np.float64) * deg, s, rtol=0, atol=2e-6 * np.maximum(1.0, np.abs(s)).max())
    # max of negated features is minus the min
    assert np.array_equal(oracle.aggregate_reduce(rp, ci, -X, MAX), -mn)
    # the error scale of the mean: mean of absolute values
    sa = oracle.aggregate_gcn(rp, ci, None, np.abs(X)).astype(np.float64)
    np.testing.assert_allclose(ab * deg, sa, rtol=1e-6, atol=1e-6)
    # constant features: every reduction returns the constant on non-empty rows
    C = np.full((80, 3), 2.5, dtype=np.float32)
    for op in (MAX, MIN, MEAN):
        out = oracle.aggregate_reduce(rp, ci, C, op)
        assert np.array_equal(out[deg[:, 0] > 0], C[deg[:, 0] > 0]) and not out[deg[:, 0] == 0].any()


def test_reductions_are_invariant_under_renumbering():
    rng = np.random.default_rng(6)
    rp, ci = random_sym_csr(50, 0.1, rng)
    X = rng.standard_normal((50, 5)).astype(np.float32)
    perm = rng.permutation(50).astype(np.int32)
    rp2, ci2 = oracle.apply_perm_csr(rp, ci, perm)
    Xp = oracle.permute_rows(X, perm)
    for op in (MAX, MIN):
        assert np.array_equal(oracle.aggregate_reduce(rp2, ci2, Xp, op)[perm], oracle.aggregate_reduce(rp, ci, X, op))
    np.testing.assert_allclose(oracle.aggregate_reduce(rp2, ci2, Xp, MEAN)[perm],
                               oracle.aggregate_reduce(rp, ci, X, MEAN), rtol=1e-6, atol=1e-7)
