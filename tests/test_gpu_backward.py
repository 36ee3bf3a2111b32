"""GPU parity tests of gnn_layer_backward against the oracle's chain-rule gradients."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features, glorot

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev


def _directed(n, avg, seed):
    """Non-symmetric random CSR with sorted duplicate-free rows (the transpose really differs)."""
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, size=int(n * avg))
    dst = rng.integers(0, n, size=int(n * avg))
    keep = src != dst
    key = np.unique(src[keep].astype(np.int64) * n + dst[keep])
    rows = (key // n).astype(np.int64)
    ci = (key % n).astype(np.int32)
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=rp[1:])
    return rp.astype(np.int32), ci


def _graph(name):
    if name == "directed":
        return _directed(3000, 6.0, 1)
    if name == "powerlaw":
        g = config_graph(2, shrink=4)
        return g.rowptr, g.colidx
    if name == "rmat":
        g = config_graph(5, shrink=64)
        return g.rowptr, g.colidx
    raise ValueError(name)


def _run_backward(kind, rp, ci, ew, eps, P, W, relu, Y, dY, want_dx=True, want_db=True, flags=0):
    n, K = P.shape
    M = W.shape[1]
    if ew is None:
        rp_t, ci_t = gnn.gnn_csr_transpose(rp, ci)
        ew_t = None
    else:
        rp_t, ci_t, ew_t = gnn.gnn_csr_transpose(rp, ci, ew)
    G = DeviceGraph(rp_t, ci_t, ew_t)
    nbytes = gnn.gnn_backward_workspace_bytes(n, G.nnz, K, M, 0)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dX = torch.full((n, K), float("nan"), device="cuda") if want_dx else None
    dW = torch.full((K, M), float("nan"), device="cuda")
    db = torch.full((M,), float("nan"), device="cuda") if want_db else None
    gnn.gnn_layer_backward(kind, n, G.nnz, G.rowptr, G.colidx, G.ew, eps, dev(P), K, dev(W), M, relu, dev(Y), dev(dY),
                           dX, dW, db, 0, 0, 0, flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    return (None if dX is None else dX.cpu().numpy()), dW.cpu().numpy(), (None if db is None else db.cpu().numpy())


@pytest.mark.parametrize("name", ["directed", "powerlaw", "rmat"])
@pytest.mark.parametrize("K,M,relu", [(40, 24, True), (64, 64, True), (96, 16, False), (16, 3, True), (7, 70, False)])
def test_gcn_layer_backward_parity(name, K, M, relu):
    rp, ci = _graph(name)
    n = rp.size - 1
    rng = np.random.default_rng(K * 100 + M)
    ew = rng.uniform(0.1, 1.0, ci.size).astype(np.float32)  # not symmetric: the transpose must carry the weights
    X = features(n, K, seed=K)
    W = glorot(K, M, seed=M)
    Y = oracle.gcn_layer(rp, ci, ew, X, W, None, relu)
    dY = features(n, M, seed=K + M)
    (rX, rW, rb), (sX, sW, sb) = oracle.gcn_layer_backward(rp, ci, ew, X, W, relu, Y, dY, want_abs=True)
    dX, dW, db = _run_backward(gnn.GNN_GCN, rp, ci, ew, 0.0, X, W, relu, Y, dY)
    assert_parity(dX, rX, sX, f"gcn dX {name}")
    assert_parity(dW, rW, sW, f"gcn dW {name}")
    assert_parity(db, rb, sb, f"gcn db {name}")


@pytest.mark.parametrize("name", ["directed", "powerlaw", "rmat"])
@pytest.mark.parametrize("K,M,relu,eps", [(64, 64, True, 0.0), (40, 24, False, 0.5), (16, 96, True, -0.25)])
def test_gin_layer_backward_parity(name, K, M, relu, eps):
    rp, ci = _graph(name)
    n = rp.size - 1
    X = features(n, K, seed=K + 1)
    W = glorot(K, M, seed=M + 1)
    A = oracle.aggregate_gin(rp, ci, eps, X)
    Y = oracle.gemm_bias_act(A, W, None, relu)
    dY = features(n, M, seed=K + M + 1)
    (rX, rW, rb), (sX, sW, sb) = oracle.gin_layer_backward(rp, ci, eps, A, W, relu, Y, dY, want_abs=True)
    dX, dW, db = _run_backward(gnn.GNN_GIN, rp, ci, None, eps, A, W, relu, Y, dY)
    assert_parity(dX, rX, sX, f"gin dX {name}")
    assert_parity(dW, rW, sW, f"gin dW {name}")
    assert_parity(db, rb, sb, f"gin db {name}")


@pytest.mark.parametrize("kind", ["gcn", "gin"])
@pytest.mark.parametrize("n,K,M,relu", [(1, 64, 64, True), (17, 36, 64, True), (1000, 64, 40, False), (4099, 48, 52, True),
                                        (70001, 64, 64, True), (33000, 60, 36, False)])
def test_widths_that_take_the_one_pass_update_backward(kind, n, K, M, relu):
    # widths in (32, 64] that are multiples of 4: dW, db and the input gradient of the Update come from one
    # kernel that never stores the masked gradient; row counts with ragged 16-row chunks and idle blocks
    rp, ci = _directed(n, 4.0, n)
    rng = np.random.default_rng(n + K)
    X = features(n, K, seed=K + 5)
    W = glorot(K, M, seed=M + 5)
    dY = features(n, M, seed=K + M + 5)
    if kind == "gcn":
        ew = rng.uniform(0.1, 1.0, ci.size).astype(np.float32)
        Y = oracle.gcn_layer(rp, ci, ew, X, W, None, relu)
        refs, scales = oracle.gcn_layer_backward(rp, ci, ew, X, W, relu, Y, dY, want_abs=True)
        got = _run_backward(gnn.GNN_GCN, rp, ci, ew, 0.0, X, W, relu, Y, dY)
    else:
        A = oracle.aggregate_gin(rp, ci, 0.25, X)
        Y = oracle.gemm_bias_act(A, W, None, relu)
        refs, scales = oracle.gin_layer_backward(rp, ci, 0.25, A, W, relu, Y, dY, want_abs=True)
        got = _run_backward(gnn.GNN_GIN, rp, ci, None, 0.25, A, W, relu, Y, dY)
    for g, r, sc, name in zip(got, refs, scales, ("dX", "dW", "db")):
        assert_parity(g, r, sc, f"{kind} {name} n {n} {K}->{M}")


def test_one_pass_update_backward_is_exact_on_integer_data():
    # small integers: every product and sum is exact in fp32, so a misplaced row, column or mask bit shows as a
    # whole number and cannot hide inside the tolerance
    n, K, M = 5000, 64, 64
    rp, ci = _directed(n, 3.0, 7)
    rng = np.random.default_rng(3)
    A = rng.integers(-3, 4, size=(n, K)).astype(np.float32)
    W = rng.integers(-2, 3, size=(K, M)).astype(np.float32)
    dY = rng.integers(-3, 4, size=(n, M)).astype(np.float32)
    Y = oracle.gemm_bias_act(A, W, None, True)
    (rX, rW, rb), _ = oracle.gin_layer_backward(rp, ci, 0.0, A, W, True, Y, dY, want_abs=True)
    dX, dW, db = _run_backward(gnn.GNN_GIN, rp, ci, None, 0.0, A, W, True, Y, dY)
    assert np.array_equal(dW, rW.astype(np.float32)) and np.array_equal(db, rb.astype(np.float32))
    assert np.array_equal(dX, rX.astype(np.float32))
    # without the optional outputs (the first layer of a model wants neither dX nor, here, db)
    none_x, dW2, none_b = _run_backward(gnn.GNN_GIN, rp, ci, None, 0.0, A, W, True, Y, dY, want_dx=False, want_db=False)
    assert none_x is None and none_b is None and np.array_equal(dW2, dW)


def test_backward_without_optional_outputs_and_on_a_symmetric_graph():
    # a symmetric graph with symmetric weights is its own transpose: the forward CSR can be passed as is
    g = config_graph(4, shrink=32)
    rp, ci = g.rowptr, g.colidx
    ew = oracle.gcn_norm(rp, ci)
    n = g.n
    X = features(n, 96, seed=5)
    W = glorot(96, 16, seed=6)
    Y = oracle.gcn_layer(rp, ci, ew, X, W, None, True)
    dY = features(n, 16, seed=7)
    (rX, rW, rb), (sX, sW, sb) = oracle.gcn_layer_backward(rp, ci, ew, X, W, True, Y, dY, want_abs=True)
    G = DeviceGraph(rp, ci, ew)
    ws = torch.empty(gnn.gnn_backward_workspace_bytes(n, G.nnz, 96, 16, 0), dtype=torch.uint8, device="cuda")
    dW = torch.empty(96, 16, device="cuda")
    gnn.gnn_layer_backward(gnn.GNN_GCN, n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 96, dev(W), 16, True, dev(Y),
                           dev(dY), None, dW, None, 0, 0, 0, 0, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    assert_parity(dW.cpu().numpy(), rW, sW, "dW only")
    with pytest.raises(gnn.GnnError):
        gnn.gnn_layer_backward(gnn.GNN_GCN, n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 96, dev(W), 16, True,
                               dev(Y), dev(dY), None, dW, None, 0, 0, 0, 0, ws[:4096])


def test_config5_one_gin_layer_backward_full_size():
    g = config_graph(5)
    n = g.n
    X = features(n, 64, seed=11)
    W = glorot(64, 64, seed=12)
    A = oracle.aggregate_gin(g.rowptr, g.colidx, 0.0, X)
    Y = oracle.gemm_bias_act(A, W, None, True)
    dY = features(n, 64, seed=13)
    (rX, rW, rb), (sX, sW, sb) = oracle.gin_layer_backward(g.rowptr, g.colidx, 0.0, A, W, True, Y, dY, want_abs=True)
    dX, dW, db = _run_backward(gnn.GNN_GIN, g.rowptr, g.colidx, None, 0.0, A, W, True, Y, dY)
    assert_parity(dX, rX, sX, "config 5 dX")
    assert_parity(dW, rW, sW, "config 5 dW")
    assert_parity(db, rb, sb, "config 5 db")


@pytest.mark.parametrize("kind", ["gcn", "gin"])
def test_deterministic_backward_is_bitwise_reproducible(kind):
    rp, ci = _graph("rmat")
    n = rp.size - 1
    K, M = 64, 32
    X = features(n, K, seed=11)
    W = glorot(K, M, seed=12)
    dY = features(n, M, seed=13)
    if kind == "gcn":
        ew = np.random.default_rng(14).uniform(0.1, 1.0, ci.size).astype(np.float32)
        Y = oracle.gcn_layer(rp, ci, ew, X, W, None, True)
        (rX, rW, rb), (sX, sW, sb) = oracle.gcn_layer_backward(rp, ci, ew, X, W, True, Y, dY, want_abs=True)
        runs = [_run_backward(gnn.GNN_GCN, rp, ci, ew, 0.0, X, W, True, Y, dY, flags=gnn.GNN_FLAG_DETERMINISTIC)
                for _ in range(3)]
    else:
        A = oracle.aggregate_gin(rp, ci, 0.0, X)
        Y = oracle.gemm_bias_act(A, W, None, True)
        (rX, rW, rb), (sX, sW, sb) = oracle.gin_layer_backward(rp, ci, 0.0, A, W, True, Y, dY, want_abs=True)
        runs = [_run_backward(gnn.GNN_GIN, rp, ci, None, 0.0, A, W, True, Y, dY, flags=gnn.GNN_FLAG_DETERMINISTIC)
                for _ in range(3)]
    assert_parity(runs[0][0], rX, sX, f"deterministic {kind} dX")
    assert_parity(runs[0][1], rW, sW, f"deterministic {kind} dW")
    assert_parity(runs[0][2], rb, sb, f"deterministic {kind} db")
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
