"""Pins for the oracle's layer and model compositions (oracle/__init__.py) and for the bias/activation
step: dense fp64 expressions written out with numpy on small graphs, values worked by hand, and
properties that single out one plausible mistake each (bias on the wrong side of the aggregation,
activation before the bias, activation after the last layer, a dropped absolute value in a scale).

Readings pinned here: a GCN layer is act(A_hat (X W) + b), the bias after the aggregation (Sec. 2.1
gives the Update as w.a + b, Eq. 2 has no bias); a GIN layer is act(((1+eps) X + sum_N X) W + b)
(Eq. 3 with one linear layer as h); a model applies ReLU after every layer but the last and no
softmax (Sec. 7.1 fixes only depth and width)."""
import numpy as np
import pytest

import oracle
from util import dense_from_csr, random_sym_csr


def _case(seed, n=23, k=7, m=5, self_loops=True, p=0.25):
    rng = np.random.default_rng(seed)
    rp, ci = random_sym_csr(n, p, rng, self_loops=self_loops)
    X = rng.standard_normal((n, k)).astype(np.float32)
    W = rng.standard_normal((k, m)).astype(np.float32)
    b = rng.standard_normal(m).astype(np.float32)
    return rng, rp, ci, X, W, b


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ---------------------------------------------------------------- bias + activation
def test_bias_act_values_worked_by_hand():
    Z = np.array([[1.0, -2.0, 0.25], [-0.5, 3.0, -4.0]], dtype=np.float32)
    b = np.array([0.5, 1.0, -1.0], dtype=np.float32)
    # Z + b = [[1.5, -1, -0.75], [0, 4, -5]]
    assert oracle.bias_act(Z, b, False).tolist() == [[1.5, -1.0, -0.75], [0.0, 4.0, -5.0]]
    assert oracle.bias_act(Z, b, True).tolist() == [[1.5, 0.0, 0.0], [0.0, 4.0, 0.0]]
    # without bias: only the activation; without either: the input itself
    assert oracle.bias_act(Z, None, True).tolist() == [[1.0, 0.0, 0.25], [0.0, 3.0, 0.0]]
    assert np.array_equal(oracle.bias_act(Z, None, False), Z)
    # the activation sees the biased value: relu(-2 + 3) = 1, not relu(-2) + 3 = 3
    assert oracle.bias_act(np.array([[-2.0]], np.float32), np.array([3.0], np.float32), True).tolist() == [[1.0]]


def test_bias_is_broadcast_over_rows_not_columns():
    Z = np.zeros((4, 3), dtype=np.float32)
    b = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    assert np.array_equal(oracle.bias_act(Z, b, False), np.tile(b, (4, 1)))


# ---------------------------------------------------------------- one layer against the dense expression
@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("relu", [False, True])
def test_gcn_layer_with_bias_equals_the_dense_expression(seed, relu):
    rng, rp, ci, X, W, b = _case(seed)
    ew = oracle.gcn_norm(rp, ci)
    A = dense_from_csr(rp, ci, ew)
    ref = A @ (_f64(X) @ _f64(W)) + _f64(b)
    if relu:
        ref = np.maximum(ref, 0.0)
    got = oracle.gcn_layer(rp, ci, ew, X, W, b, relu)
    assert got.dtype == np.float32
    # (the oracle stores X W as float between the two operations: a few float roundings apart)
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    # the bias is added after the aggregation: A_hat (X W + b) differs by (rowsum(A_hat) - 1) b
    wrong = A @ (_f64(X) @ _f64(W) + _f64(b))
    if relu:
        wrong = np.maximum(wrong, 0.0)
    assert np.abs(got - wrong).max() > 1e-2
    if relu:
        assert (got >= 0).all() and (got == 0).any()
    else:
        assert (got < 0).any()


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("relu", [False, True])
def test_gin_layer_with_bias_equals_the_dense_expression(seed, relu):
    rng, rp, ci, X, W, b = _case(10 + seed, self_loops=False)
    eps = 0.25
    A = dense_from_csr(rp, ci) + (1.0 + eps) * np.eye(rp.size - 1)
    ref = (A @ _f64(X)) @ _f64(W) + _f64(b)
    if relu:
        ref = np.maximum(ref, 0.0)
    got = oracle.gin_layer(rp, ci, eps, X, W, b, relu)
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    # the self term carries 1 + eps, and the bias enters once per output row
    no_eps = ((dense_from_csr(rp, ci) + np.eye(rp.size - 1)) @ _f64(X)) @ _f64(W) + _f64(b)
    assert np.abs(got - (np.maximum(no_eps, 0.0) if relu else no_eps)).max() > 1e-2


def test_layers_without_bias_are_the_layers_with_a_zero_bias():
    _, rp, ci, X, W, _ = _case(3)
    ew = oracle.gcn_norm(rp, ci)
    z = np.zeros(W.shape[1], dtype=np.float32)
    assert np.array_equal(oracle.gcn_layer(rp, ci, ew, X, W, None, True), oracle.gcn_layer(rp, ci, ew, X, W, z, True))
    assert np.array_equal(oracle.gin_layer(rp, ci, 0.0, X, W, None, True), oracle.gin_layer(rp, ci, 0.0, X, W, z, True))


# ---------------------------------------------------------------- models: ReLU after every layer but the last
def _dense_chain(A, X, Ws, bs, gcn):
    H = _f64(X)
    for l, W in enumerate(Ws):
        Z = A @ (H @ _f64(W)) if gcn else (A @ H) @ _f64(W)
        if bs is not None and bs[l] is not None:
            Z = Z + _f64(bs[l])
        H = Z if l == len(Ws) - 1 else np.maximum(Z, 0.0)
    return H


@pytest.mark.parametrize("with_bias", [False, True])
def test_gcn_model_of_three_layers_equals_the_dense_chain(with_bias):
    rng, rp, ci, X, _, _ = _case(21, n=31, k=9, p=0.06)
    dims = [9, 6, 5, 4]
    Ws = [rng.standard_normal((dims[i], dims[i + 1])).astype(np.float32) for i in range(3)]
    bs = [rng.standard_normal(dims[i + 1]).astype(np.float32) for i in range(3)] if with_bias else None
    ew = oracle.gcn_norm(rp, ci)
    A = dense_from_csr(rp, ci, ew)
    ref = _dense_chain(A, X, Ws, bs, gcn=True)
    got = oracle.gcn_model(rp, ci, ew, X, Ws, bs)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    assert (got < 0).any(), "the last layer must not be activated"
    # an activation after the last layer, or none between the layers, is a different function
    assert np.abs(got - np.maximum(ref, 0.0)).max() > 1e-2
    H = _f64(X)
    for l, W in enumerate(Ws):
        H = A @ (H @ _f64(W)) + (0.0 if bs is None else _f64(bs[l]))
    assert np.abs(got - H).max() > 1e-2 * np.abs(H).max()
    # the model is its layers chained
    step = X
    for l, W in enumerate(Ws):
        step = oracle.gcn_layer(rp, ci, ew, step, W, None if bs is None else bs[l], relu=l != 2)
    assert np.array_equal(got, step)


@pytest.mark.parametrize("with_bias", [False, True])
def test_gin_model_of_three_layers_equals_the_dense_chain(with_bias):
    rng, rp, ci, X, _, _ = _case(22, n=29, k=8, self_loops=False, p=0.15)
    dims = [8, 8, 8, 3]
    Ws = [(0.4 * rng.standard_normal((dims[i], dims[i + 1]))).astype(np.float32) for i in range(3)]
    bs = [rng.standard_normal(dims[i + 1]).astype(np.float32) for i in range(3)] if with_bias else None
    eps = -0.5
    A = dense_from_csr(rp, ci) + (1.0 + eps) * np.eye(rp.size - 1)
    ref = _dense_chain(A, X, Ws, bs, gcn=False)
    got = oracle.gin_model(rp, ci, eps, X, Ws, bs)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    assert (got < 0).any()
    assert np.abs(got - np.maximum(ref, 0.0)).max() > 1e-2
    step = X
    for l, W in enumerate(Ws):
        step = oracle.gin_layer(rp, ci, eps, step, W, None if bs is None else bs[l], relu=l != 2)
    assert np.array_equal(got, step)


def test_model_error_scale_is_the_last_layers():
    rng, rp, ci, X, _, _ = _case(23, n=19, k=6)
    Ws = [rng.standard_normal((6, 6)).astype(np.float32) for _ in range(2)]
    ew = oracle.gcn_norm(rp, ci)
    out, scale = oracle.gcn_model(rp, ci, ew, X, Ws, None, want_abs=True)
    H1 = oracle.gcn_layer(rp, ci, ew, X, Ws[0], None, relu=True)
    out2, scale2 = oracle.gcn_layer(rp, ci, ew, H1, Ws[1], None, relu=False, want_abs=True)
    assert np.array_equal(out, out2) and np.array_equal(scale, scale2)


# ---------------------------------------------------------------- the error scales of the layer parity gates
@pytest.mark.parametrize("seed", range(3))
def test_gcn_layer_error_scale_equals_the_dense_expression(seed):
    rng, rp, ci, X, W, b = _case(30 + seed)
    ew = oracle.gcn_norm(rp, ci)
    ew[::3] *= -1.0  # signs must not matter: every factor enters by its absolute value
    Aabs = dense_from_csr(rp, ci, np.abs(ew))
    want = Aabs @ (np.abs(_f64(X)) @ np.abs(_f64(W))) + np.abs(_f64(b))
    out, scale, last = oracle.gcn_layer(rp, ci, ew, X, W, b, True, want_abs="both")
    assert scale.dtype == np.float64
    np.testing.assert_allclose(scale, want, rtol=1e-12, atol=0)
    # without a bias its term is absent
    _, scale0 = oracle.gcn_layer(rp, ci, ew, X, W, None, True, want_abs=True)
    np.testing.assert_allclose(scale0, want - np.abs(_f64(b)), rtol=1e-12, atol=1e-300)
    # the stricter scale of the last operation alone: |A_hat| |fl(X W)| + |b|, never above the full one
    H = oracle.gemm_bias_act(X, W)
    np.testing.assert_allclose(last, Aabs @ np.abs(_f64(H)) + np.abs(_f64(b)), rtol=1e-12, atol=0)
    assert (last <= scale * (1 + 1e-6)).all() and (last < 0.9 * scale).any()
    # and both bound the value they guard
    assert (np.abs(_f64(out)) <= last * (1 + 1e-6)).all()


@pytest.mark.parametrize("seed", range(3))
def test_gin_layer_error_scale_equals_the_dense_expression(seed):
    rng, rp, ci, X, W, b = _case(40 + seed, self_loops=False)
    eps = -1.75  # |1 + eps| = 0.75: the absolute value of the self factor must be taken
    A = dense_from_csr(rp, ci)
    want = (abs(1.0 + eps) * np.abs(_f64(X)) + A @ np.abs(_f64(X))) @ np.abs(_f64(W)) + np.abs(_f64(b))
    out, scale, last = oracle.gin_layer(rp, ci, eps, X, W, b, False, want_abs="both")
    np.testing.assert_allclose(scale, want, rtol=1e-12, atol=0)
    agg = oracle.aggregate_gin(rp, ci, eps, X)
    np.testing.assert_allclose(last, np.abs(_f64(agg)) @ np.abs(_f64(W)) + np.abs(_f64(b)), rtol=1e-12, atol=0)
    assert (last <= scale * (1 + 1e-6)).all() and (last < 0.9 * scale).any()
    assert (np.abs(_f64(out)) <= last * (1 + 1e-6)).all()


def test_aggregation_error_scales_are_the_sums_of_absolute_terms():
    rng, rp, ci, X, _, _ = _case(50)
    ew = oracle.gcn_norm(rp, ci)
    ew[1::2] *= -1.0
    _, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    np.testing.assert_allclose(ab, dense_from_csr(rp, ci, np.abs(ew)) @ np.abs(_f64(X)), rtol=1e-12)
    _, ab = oracle.aggregate_gin(rp, ci, -3.0, X, want_abs=True)
    np.testing.assert_allclose(ab, (dense_from_csr(rp, ci) + 2.0 * np.eye(rp.size - 1)) @ np.abs(_f64(X)), rtol=1e-12)
    A = rng.standard_normal((11, 6)).astype(np.float32)
    W = rng.standard_normal((6, 4)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    _, ab = oracle.gemm_bias_act(A, W, b, True, want_abs=True)
    np.testing.assert_allclose(ab, np.abs(_f64(A)) @ np.abs(_f64(W)) + np.abs(_f64(b)), rtol=1e-12)


def test_row_partitioned_forms_equal_the_single_thread_functions_bit_for_bit():
    """The benchmark's all-cores baseline runs the same C loops on disjoint row ranges."""
    from gnn_synth import config_graph, features, glorot
    g = config_graph(2, shrink=4)
    X = features(g.n, 24, seed=1)
    W = glorot(24, 10, seed=2)
    b = features(1, 10, seed=3)[0]
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    for threads in (1, 3, 8):
        assert np.array_equal(oracle.gcn_layer_threads(g.rowptr, g.colidx, ew, X, W, b, True, threads),
                              oracle.gcn_layer(g.rowptr, g.colidx, ew, X, W, b, True))
        assert np.array_equal(oracle.gin_layer_threads(g.rowptr, g.colidx, 0.5, X, W, b, True, threads),
                              oracle.gin_layer(g.rowptr, g.colidx, 0.5, X, W, b, True))
        assert np.array_equal(oracle.aggregate_gcn_threads(g.rowptr, g.colidx, ew, X, threads),
                              oracle.aggregate_gcn(g.rowptr, g.colidx, ew, X))
    g5 = config_graph(5, shrink=64)  # many rows without entries
    X5 = features(g5.n, 8, seed=4)
    W5 = glorot(8, 8, seed=5)
    assert np.array_equal(oracle.gin_layer_threads(g5.rowptr, g5.colidx, 0.0, X5, W5, None, False, 5),
                          oracle.gin_layer(g5.rowptr, g5.colidx, 0.0, X5, W5, None, False))
