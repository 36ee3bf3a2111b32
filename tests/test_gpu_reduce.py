"""GPU parity tests of gnn_aggregate_reduce (max / min / mean / unweighted sum over neighbours).

Max and min involve no rounding, so the GPU must reproduce the oracle bit for bit; mean is held to
the 1e-5 gates of the sum it is made of."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features
from util import csr_from_edges

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev


def _graph(kind):
    if kind == "powerlaw":
        g = config_graph(2, shrink=4)
        return g.rowptr, g.colidx
    if kind == "rmat":
        g = config_graph(5, shrink=64)  # many rows without entries
        return g.rowptr, g.colidx
    if kind == "star":
        n = 6001
        return csr_from_edges(n, [(0, i) for i in range(1, n)], self_loops=True)
    raise ValueError(kind)


def _run(op, G, X, ngs=0, dw=0, wpb=0, flags=0, ws=None):
    Xd = dev(X)
    out = torch.full_like(Xd, float("nan"))
    if ws is None:
        ws = gnn.alloc_workspace(G.n, G.nnz, X.shape[1], ngs)
    gnn.gnn_aggregate_reduce(op, G.n, G.nnz, G.rowptr, G.colidx, Xd, out, X.shape[1], ngs, dw, wpb, flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    return out.cpu().numpy()


@pytest.mark.parametrize("kind", ["powerlaw", "rmat", "star"])
@pytest.mark.parametrize("dim,ngs,dw,wpb", [(64, 0, 0, 0), (16, 4, 4, 4), (22, 8, 0, 0), (3, 2, 1, 2), (96, 16, 8, 3),
                                            (130, 8, 64, 0), (64, 2, 16, 8)])
def test_max_min_are_bit_exact_and_mean_sum_within_tolerance(kind, dim, ngs, dw, wpb):
    rp, ci = _graph(kind)
    n = rp.size - 1
    X = features(n, dim, seed=700 + dim)
    G = DeviceGraph(rp, ci)
    ws = gnn.alloc_workspace(G.n, G.nnz, dim, ngs)
    for op, oop in ((gnn.GNN_REDUCE_MAX, oracle.REDUCE_MAX), (gnn.GNN_REDUCE_MIN, oracle.REDUCE_MIN)):
        got = _run(op, G, X, ngs, dw, wpb, ws=ws)
        ref = oracle.aggregate_reduce(rp, ci, X, oop)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"op {op} {kind} dim {dim}"
    ref, ab = oracle.aggregate_reduce(rp, ci, X, oracle.REDUCE_MEAN, want_abs=True)
    assert_parity(_run(gnn.GNN_REDUCE_MEAN, G, X, ngs, dw, wpb, ws=ws), ref, ab, f"mean {kind} dim {dim}")
    ref, ab = oracle.aggregate_gcn(rp, ci, None, X, want_abs=True)
    assert_parity(_run(gnn.GNN_REDUCE_SUM, G, X, ngs, dw, wpb, ws=ws), ref, ab, f"sum {kind} dim {dim}")


def test_reduce_on_degenerate_inputs_and_argument_errors():
    # no entries at all: every reduction gives zeros
    rp = np.zeros(6, dtype=np.int32)
    ci = np.zeros(0, dtype=np.int32)
    X = features(5, 8, seed=1)
    G = DeviceGraph(rp, ci)
    for op in (gnn.GNN_REDUCE_MAX, gnn.GNN_REDUCE_MIN, gnn.GNN_REDUCE_MEAN, gnn.GNN_REDUCE_SUM):
        assert not _run(op, G, X).any()
    # negative-only features: the maximum of a non-empty row stays negative, an empty row gives 0
    rp2, ci2 = csr_from_edges(6, [(0, 1), (1, 2), (3, 4)])
    Xn = -np.abs(features(6, 4, seed=2)) - 1.0
    G2 = DeviceGraph(rp2, ci2)
    got = _run(gnn.GNN_REDUCE_MAX, G2, Xn)
    assert np.array_equal(got, oracle.aggregate_reduce(rp2, ci2, Xn, oracle.REDUCE_MAX))
    assert (got[:5] < 0).all() and not got[5].any()
    # refusals
    Xd = dev(X)
    out = torch.empty_like(Xd)
    with pytest.raises(gnn.GnnError) as e:  # unknown op
        gnn.gnn_aggregate_reduce(7, G.n, G.nnz, G.rowptr, G.colidx, Xd, out, 8, 0, 0, 0, 0, gnn.alloc_workspace(5, 0, 8, 0))
    assert e.value.code == -1
    with pytest.raises(gnn.GnnError) as e:  # max needs the rows for partial results
        gnn.gnn_aggregate_reduce(gnn.GNN_REDUCE_MAX, G2.n, G2.nnz, G2.rowptr, G2.colidx, dev(Xn), torch.empty(6, 4, device="cuda"),
                                 4, 0, 0, 0, 0, gnn.alloc_workspace(6, G2.nnz, 0, 0))
    assert e.value.code == -3
    with pytest.raises(gnn.GnnError) as e:  # no atomic flush for max
        gnn.gnn_aggregate_reduce(gnn.GNN_REDUCE_MAX, G2.n, G2.nnz, G2.rowptr, G2.colidx, dev(Xn), torch.empty(6, 4, device="cuda"),
                                 4, 0, 0, 0, gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.alloc_workspace(6, G2.nnz, 4, 0))
    assert e.value.code == -1


def test_reduce_full_size_rmat():
    """Configuration 5 at full size: hubs whose groups span dozens of blocks, half the rows empty."""
    g = config_graph(5)
    X = features(g.n, 64, seed=9)
    G = DeviceGraph(g.rowptr, g.colidx)
    ws = gnn.alloc_workspace(G.n, G.nnz, 64, 0)
    got = _run(gnn.GNN_REDUCE_MAX, G, X, ws=ws)
    assert np.array_equal(got.view(np.uint32), oracle.aggregate_reduce(g.rowptr, g.colidx, X, oracle.REDUCE_MAX).view(np.uint32))
    ref, ab = oracle.aggregate_reduce(g.rowptr, g.colidx, X, oracle.REDUCE_MEAN, want_abs=True)
    assert_parity(_run(gnn.GNN_REDUCE_MEAN, G, X, ws=ws), ref, ab, "mean config 5")
