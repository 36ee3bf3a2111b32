"""Seeded random graphs and parameter combinations through the entry points whose other tests use fixed
cases: gnn_aggregate_reduce, gnn_aggregate_edge, gnn_aggregate_gin_static, gnn_layer_forward (both kinds, every
flag that changes the path) and gnn_layer_backward.  A refusal must be one of the two documented ones (a block's
scratch memory above the limit, or no room for partial rows in the workspace)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import features, glorot
from util import parity_errors

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import TOL, DeviceGraph, dev

DIMS = [1, 2, 3, 4, 5, 8, 16, 22, 31, 32, 64, 96, 100, 128, 200]


def _random_graph(rng):
    """Empty rows, short rows and up to two rows long enough to span many blocks; duplicates allowed."""
    n = int(rng.integers(1, 700))
    deg = rng.choice([0, 1, 2, 3, 5, 9, 17, 40], size=n, p=[0.2, 0.2, 0.15, 0.15, 0.1, 0.1, 0.05, 0.05])
    for _ in range(int(rng.integers(0, 3))):
        deg[int(rng.integers(0, n))] = int(rng.integers(100, 3000))
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    return rp, rng.integers(0, n, size=int(rp[-1])).astype(np.int32)


def _params(rng):
    return (int(rng.choice([0, 0, 1, 2, 3, 4, 7, 8, 16, 32, 64])), int(rng.choice([0, 0, 1, 2, 4, 8, 16, 32, 64])),
            int(rng.choice([0, 0, 1, 2, 3, 4, 8, 16])))


def _check(got, ref, scale, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    normwise, guarded = parity_errors(got, ref, scale)
    assert guarded <= TOL, f"{what}: guarded componentwise error {guarded:.3e}"
    # on an output of a handful of numbers the normwise measure is the relative error of one cancelling sum
    assert normwise <= TOL or got.size < 64, f"{what}: normwise error {normwise:.3e}"


def _refusal_is_documented(e, what):
    assert e.code in (-5, -3), f"{what}: refused with code {e.code}"


@pytest.mark.parametrize("seed", range(40))
def test_reduce(seed):
    rng = np.random.default_rng(91000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    ngs, dw, wpb = _params(rng)
    dim = int(rng.choice(DIMS))
    flags = int(rng.choice([0, 0, gnn.GNN_FLAG_XCD_RUNS, gnn.GNN_FLAG_DETERMINISTIC]))
    what = f"reduce seed {seed}: n {n} nnz {nnz} dim {dim} ngs {ngs} dw {dw} wpb {wpb} flags {flags}"
    print(what, flush=True)
    X = features(n, dim, seed=seed)
    G = DeviceGraph(rp, ci)
    ws = gnn.alloc_workspace(n, nnz, 4 * dim, ngs)
    for op, oop in ((gnn.GNN_REDUCE_SUM, None), (gnn.GNN_REDUCE_MEAN, oracle.REDUCE_MEAN),
                    (gnn.GNN_REDUCE_MAX, oracle.REDUCE_MAX), (gnn.GNN_REDUCE_MIN, oracle.REDUCE_MIN)):
        out = torch.full((n, dim), float("nan"), device="cuda")
        try:
            gnn.gnn_aggregate_reduce(op, n, nnz, G.rowptr, G.colidx, dev(X), out, dim, ngs, dw, wpb, flags, ws)
        except gnn.GnnError as e:
            return _refusal_is_documented(e, what)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        got = out.cpu().numpy()
        if op in (gnn.GNN_REDUCE_MAX, gnn.GNN_REDUCE_MIN):
            ref = oracle.aggregate_reduce(rp, ci, X, oop)
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"{what} op {op}"
        elif op == gnn.GNN_REDUCE_MEAN:
            _check(got, *oracle.aggregate_reduce(rp, ci, X, oop, want_abs=True), what + " mean")
        else:
            _check(got, *oracle.aggregate_gcn(rp, ci, None, X, want_abs=True), what + " sum")


@pytest.mark.parametrize("seed", range(40))
def test_edge_vectors(seed):
    rng = np.random.default_rng(92000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    ngs, dw, wpb = _params(rng)
    dim = int(rng.choice(DIMS))
    flags = int(rng.choice([0, 0, gnn.GNN_FLAG_XCD_RUNS, gnn.GNN_FLAG_DETERMINISTIC]))
    what = f"edge vectors seed {seed}: n {n} nnz {nnz} dim {dim} ngs {ngs} dw {dw} wpb {wpb} flags {flags}"
    print(what, flush=True)
    X = features(n, dim, seed=seed)
    E = features(nnz, dim, seed=seed + 1) if nnz else np.zeros((0, dim), dtype=np.float32)
    G = DeviceGraph(rp, ci)
    ws = gnn.alloc_workspace(n, nnz, 4 * dim, ngs)
    out = torch.full((n, dim), float("nan"), device="cuda")
    try:
        gnn.gnn_aggregate_edge(n, nnz, G.rowptr, G.colidx, dev(E) if nnz else torch.zeros(1, dim, device="cuda"), dev(X),
                               out, dim, ngs, dw, wpb, flags, ws)
    except gnn.GnnError as e:
        return _refusal_is_documented(e, what)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    _check(out.cpu().numpy(), *oracle.aggregate_edge_vec(rp, ci, E, X, want_abs=True), what)


@pytest.mark.parametrize("seed", range(40))
def test_static_scratch(seed):
    rng = np.random.default_rng(93000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    ngs, dw, wpb = _params(rng)
    dim = int(rng.choice(DIMS))
    eps = float(rng.choice([0.0, 0.5, -1.0]))
    flags = int(rng.choice([0, 0, gnn.GNN_FLAG_XCD_RUNS, gnn.GNN_FLAG_DETERMINISTIC, gnn.GNN_FLAG_ATOMIC_FLUSH]))
    what = f"static scratch seed {seed}: n {n} nnz {nnz} dim {dim} ngs {ngs} dw {dw} wpb {wpb} flags {flags}"
    print(what, flush=True)
    X = features(n, dim, seed=seed)
    G = DeviceGraph(rp, ci)
    out = torch.full((n, dim), float("nan"), device="cuda")
    try:
        scratch = gnn.gnn_aggregate_gin_static(n, nnz, G.rowptr, G.colidx, eps, dev(X), out, dim, ngs, dw, wpb, flags)
    except gnn.GnnError as e:
        return _refusal_is_documented(e, what)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(scratch)
    _check(out.cpu().numpy(), *oracle.aggregate_gin(rp, ci, eps, X, want_abs=True), what)


@pytest.mark.parametrize("seed", range(60))
def test_layer_forward(seed):
    rng = np.random.default_rng(94000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    ngs, dw, wpb = _params(rng)
    K = int(rng.choice([1, 3, 5, 16, 22, 32, 64, 96, 100, 128]))
    M = int(rng.choice([1, 3, 7, 16, 22, 48, 64, 70, 100]))
    gcn, relu = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    flags = int(rng.choice([0, 0, 0, gnn.GNN_FLAG_NO_FUSION, gnn.GNN_FLAG_FUSION, gnn.GNN_FLAG_GCN_UPDATE_FIRST,
                            gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.GNN_FLAG_DETERMINISTIC, gnn.GNN_FLAG_XCD_RUNS]))
    X, W = features(n, K, seed=seed), glorot(K, M, seed=seed + 1)
    b = features(1, M, seed=seed + 2)[0] if rng.integers(0, 2) else None
    what = (f"layer seed {seed}: n {n} nnz {nnz} {'gcn' if gcn else 'gin'} {K}->{M} ngs {ngs} dw {dw} wpb {wpb} "
            f"flags {flags} relu {relu} bias {b is not None}")
    print(what, flush=True)
    if gcn:
        ew = rng.standard_normal(nnz).astype(np.float32)
        ref, scale = oracle.gcn_layer(rp, ci, ew, X, W, b, relu, want_abs=True)
        G, kind, eps = DeviceGraph(rp, ci, ew), gnn.GNN_GCN, 0.0
    else:
        eps = float(rng.choice([0.0, 0.5, -1.0]))
        ref, scale = oracle.gin_layer(rp, ci, eps, X, W, b, relu, want_abs=True)
        G, kind = DeviceGraph(rp, ci), gnn.GNN_GIN
    ws = gnn.alloc_workspace(n, nnz, 4 * max(K, M), ngs)
    out = torch.full((n, M), float("nan"), device="cuda")
    try:
        gnn.gnn_layer_forward(kind, n, nnz, G.rowptr, G.colidx, G.ew if gcn else None, eps, dev(X), K, dev(W), dev(b), M,
                              relu, out, ngs, dw, wpb, flags, ws)
    except gnn.GnnError as e:
        return _refusal_is_documented(e, what)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    _check(out.cpu().numpy(), ref, scale, what)


@pytest.mark.parametrize("seed", range(40))
def test_layer_backward(seed):
    rng = np.random.default_rng(95000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    K = int(rng.choice([1, 3, 7, 16, 40, 64, 96]))
    M = int(rng.choice([1, 3, 16, 24, 64, 70]))
    gcn, relu = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    flags = int(rng.choice([0, 0, gnn.GNN_FLAG_DETERMINISTIC]))
    X, W, dY = features(n, K, seed=seed), glorot(K, M, seed=seed + 1), features(n, M, seed=seed + 3)
    what = f"backward seed {seed}: n {n} nnz {nnz} {'gcn' if gcn else 'gin'} {K}->{M} relu {relu} flags {flags}"
    print(what, flush=True)
    if gcn:
        ew = rng.uniform(0.1, 1.0, nnz).astype(np.float32)
        P, eps, kind = X, 0.0, gnn.GNN_GCN
        Y = oracle.gcn_layer(rp, ci, ew, X, W, None, relu)
        refs, scales = oracle.gcn_layer_backward(rp, ci, ew, X, W, relu, Y, dY, want_abs=True)
        rp_t, ci_t, ew_t = gnn.gnn_csr_transpose(rp, ci, ew)
    else:
        eps, kind = float(rng.choice([0.0, 0.5, -0.25])), gnn.GNN_GIN
        P = oracle.aggregate_gin(rp, ci, eps, X)  # the GIN backward starts from the aggregated rows
        Y = oracle.gemm_bias_act(P, W, None, relu)
        refs, scales = oracle.gin_layer_backward(rp, ci, eps, P, W, relu, Y, dY, want_abs=True)
        (rp_t, ci_t), ew_t = gnn.gnn_csr_transpose(rp, ci), None
    G = DeviceGraph(rp_t, ci_t, ew_t)
    ws = torch.empty(gnn.gnn_backward_workspace_bytes(n, G.nnz, K, M, 0), dtype=torch.uint8, device="cuda")
    dX = torch.full((n, K), float("nan"), device="cuda")
    dW = torch.full((K, M), float("nan"), device="cuda")
    db = torch.full((M,), float("nan"), device="cuda")
    gnn.gnn_layer_backward(kind, n, G.nnz, G.rowptr, G.colidx, G.ew, eps, dev(P), K, dev(W), M, relu, dev(Y), dev(dY),
                           dX, dW, db, 0, 0, 0, flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    for got, ref, scale, name in zip((dX, dW, db), refs, scales, ("dX", "dW", "db")):
        _check(got.cpu().numpy(), ref, scale, f"{what} {name}")
