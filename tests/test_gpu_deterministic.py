"""The ordered flush (GNN_FLAG_DETERMINISTIC, and the default when the workspace has room): no float
atomics, so repeated runs agree bit for bit; values still match the oracle.  GNN_FLAG_ATOMIC_FLUSH
selects the atomic flush of Sec. 5.2 instead."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features, glorot
from util import csr_from_edges

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev, run_gcn, run_gin

DET = gnn.GNN_FLAG_DETERMINISTIC


def _graph(kind):
    if kind == "powerlaw":
        g = config_graph(2, shrink=4)
        return g.rowptr, g.colidx
    if kind == "rmat":
        g = config_graph(5, shrink=64)
        return g.rowptr, g.colidx
    if kind == "star":  # one row that spans every block, the rest are single entries
        n = 6001
        return csr_from_edges(n, [(0, i) for i in range(1, n)], self_loops=True)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["powerlaw", "rmat", "star"])
@pytest.mark.parametrize("dim,ngs,dw,wpb", [(64, 0, 0, 0), (16, 4, 4, 4), (64, 2, 16, 8), (22, 8, 0, 0), (3, 1, 1, 1),
                                            (96, 16, 8, 3), (130, 8, 64, 0), (64, 32, 64, 16)])
def test_repeated_runs_are_bitwise_identical_and_match_the_oracle(kind, dim, ngs, dw, wpb):
    rp, ci = _graph(kind)
    n = rp.size - 1
    X = features(n, dim, seed=900 + dim)
    ew = oracle.gcn_norm(rp, ci)
    G = DeviceGraph(rp, ci, ew)
    ws = gnn.alloc_workspace(G.n, G.nnz, dim, ngs)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    first = run_gcn(G, X, ngs=ngs, dw=dw, wpb=wpb, flags=DET, ws=ws)
    assert_parity(first, ref, ab, f"deterministic gcn {kind} dim {dim}")
    atomic = run_gcn(G, X, ngs=ngs, dw=dw, wpb=wpb, flags=gnn.GNN_FLAG_ATOMIC_FLUSH, ws=ws)  # leaves no trace
    assert_parity(atomic, ref, ab, f"atomic flush gcn {kind} dim {dim}")
    for _ in range(3):
        again = run_gcn(G, X, ngs=ngs, dw=dw, wpb=wpb, flags=DET | gnn.GNN_FLAG_REUSE_PARTITION, ws=ws)
        assert np.array_equal(first.view(np.uint32), again.view(np.uint32))
    G2 = DeviceGraph(rp, ci)
    ref, ab = oracle.aggregate_gin(rp, ci, 0.25, X, want_abs=True)
    first = run_gin(G2, 0.25, X, ngs=ngs, dw=dw, wpb=wpb, flags=DET, ws=ws)
    assert_parity(first, ref, ab, f"deterministic gin {kind} dim {dim}")
    for _ in range(3):
        again = run_gin(G2, 0.25, X, ngs=ngs, dw=dw, wpb=wpb, flags=DET, ws=ws)
        assert np.array_equal(first.view(np.uint32), again.view(np.uint32))


@pytest.mark.parametrize("kind_id", ["gcn", "gin"])
def test_deterministic_layers_with_bias_and_relu(kind_id):
    rp, ci = _graph("rmat")
    n = rp.size - 1
    K, M = 64, 48
    X = features(n, K, seed=77)
    W = glorot(K, M, seed=78)
    b = features(1, M, seed=79)[0] * 0.1
    ngs = 4  # small groups: many rows span blocks, so the second pass applies the epilogue to many rows
    if kind_id == "gcn":
        ew = oracle.gcn_norm(rp, ci)
        G = DeviceGraph(rp, ci, ew)
        ref, scale = oracle.gcn_layer(rp, ci, ew, X, W, b, True, want_abs=True)
        kind = gnn.GNN_GCN
    else:
        G = DeviceGraph(rp, ci)
        ref, scale = oracle.gin_layer(rp, ci, 0.0, X, W, b, True, want_abs=True)
        kind = gnn.GNN_GIN
    ws = gnn.alloc_workspace(G.n, G.nnz, max(K, M), ngs)
    Xd, Wd, bd = dev(X), dev(W), dev(b)
    outs = []
    for _ in range(3):
        out = torch.full((n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(kind, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, Xd, K, Wd, bd, M, True, out, ngs, 0, 0,
                              DET, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs.append(out.cpu().numpy())
    assert_parity(outs[0], ref, scale, f"deterministic {kind_id} layer")
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))
    assert np.array_equal(outs[0].view(np.uint32), outs[2].view(np.uint32))


def test_deterministic_mode_argument_errors():
    rp, ci = _graph("powerlaw")
    G = DeviceGraph(rp, ci)
    X = dev(features(G.n, 16, seed=1))
    out = torch.empty_like(X)
    small = gnn.alloc_workspace(G.n, G.nnz, 0, 8)  # sized without rows for the partial sums
    with pytest.raises(gnn.GnnError) as e:
        gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 8, 0, 0, DET, small)
    assert e.value.code == -3  # GNN_EWORKSPACE
    ws = gnn.alloc_workspace(G.n, G.nnz, 16, 8)
    for other in (gnn.GNN_FLAG_NO_BLOCK_OPT, gnn.GNN_FLAG_ATOMIC_FLUSH):
        with pytest.raises(gnn.GnnError) as e:
            gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 8, 0, 0, DET | other, ws)
        assert e.value.code == -1  # GNN_EINVAL


def test_default_is_ordered_when_the_workspace_has_room_and_atomic_otherwise():
    rp, ci = _graph("rmat")
    n = rp.size - 1
    X = features(n, 64, seed=21)
    G = DeviceGraph(rp, ci)
    ref, ab = oracle.aggregate_gin(rp, ci, 0.0, X, want_abs=True)
    roomy = gnn.alloc_workspace(G.n, G.nnz, 64, 4)
    first = run_gin(G, 0.0, X, ngs=4, ws=roomy, flags=gnn.GNN_FLAG_NO_PIPELINE)
    assert_parity(first, ref, ab, "default with room")
    required = run_gin(G, 0.0, X, ngs=4, ws=roomy, flags=gnn.GNN_FLAG_NO_PIPELINE | DET)
    assert np.array_equal(first.view(np.uint32), required.view(np.uint32))  # same flush, same bits
    for _ in range(3):
        again = run_gin(G, 0.0, X, ngs=4, ws=roomy, flags=gnn.GNN_FLAG_NO_PIPELINE)
        assert np.array_equal(first.view(np.uint32), again.view(np.uint32))
    tight = gnn.alloc_workspace(G.n, G.nnz, 0, 4)  # no rows for partial sums: the atomic flush serves
    assert_parity(run_gin(G, 0.0, X, ngs=4, ws=tight), ref, ab, "default without room")


def test_deterministic_full_size_rmat():
    """Configuration 5 at full size (hubs of up to 39,649 entries span dozens of blocks)."""
    g = config_graph(5)
    n, dim = g.n, 64
    X = features(n, dim, seed=5)
    G = DeviceGraph(g.rowptr, g.colidx)
    ws = gnn.alloc_workspace(G.n, G.nnz, dim, 0)
    first = run_gin(G, 0.0, X, flags=DET, ws=ws)
    for _ in range(2):
        again = run_gin(G, 0.0, X, flags=DET | gnn.GNN_FLAG_REUSE_PARTITION, ws=ws)
        assert np.array_equal(first.view(np.uint32), again.view(np.uint32))
    ref, ab = oracle.aggregate_gin(g.rowptr, g.colidx, 0.0, X, want_abs=True)
    assert_parity(first, ref, ab, "deterministic config 5")


def test_ordered_flush_on_two_streams_at_once():
    """Two aggregations with their own workspaces run concurrently on two streams; each must give the
    bits it gives alone (partial rows and arrival counters are per workspace)."""
    g = config_graph(5, shrink=4)
    n = g.n
    G = DeviceGraph(g.rowptr, g.colidx)
    Xa, Xb = dev(features(n, 64, seed=31)), dev(features(n, 64, seed=32))
    wsa, wsb = gnn.alloc_workspace(G.n, G.nnz, 64, 0), gnn.alloc_workspace(G.n, G.nnz, 64, 0)
    ref_a, ref_b = torch.empty_like(Xa), torch.empty_like(Xb)
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, Xa, ref_a, 64, 0, 0, 0, DET, wsa)
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, Xb, ref_b, 64, 0, 0, 0, DET, wsb)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs_a = [torch.empty_like(Xa) for _ in range(6)]
    outs_b = [torch.empty_like(Xb) for _ in range(6)]
    reuse = DET | gnn.GNN_FLAG_REUSE_PARTITION
    for oa, ob in zip(outs_a, outs_b):
        gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, Xa, oa, 64, 0, 0, 0, reuse, wsa, sa)
        gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, Xb, ob, 64, 0, 0, 0, reuse, wsb, sb)
    torch.cuda.synchronize()
    for oa, ob in zip(outs_a, outs_b):
        assert torch.equal(oa, ref_a) and torch.equal(ob, ref_b)
    gnn.gnn_workspace_status(wsa)
    gnn.gnn_workspace_status(wsb)


@pytest.mark.parametrize("dim,dw", [(64, 16), (16, 4), (96, 8), (7, 8)])
def test_every_node_spans_many_blocks_and_integer_sums_are_exact(dim, dw):
    """Sharp test of the cross-block hand-over of the ordered flush.  With one entry per group and one
    wave per block, a block serves 64/dw groups, so every node of this dense graph (rows of 128 to 223
    entries) spans at least eight blocks, which the dispatcher deals over all XCDs: every output row is
    the sum of partial rows published by other blocks.  Features and weights are small integers, so every
    partial sum is exact in fp32 and the result must equal the oracle bit for bit: a stale or torn partial
    row cannot hide in rounding."""
    rng = np.random.default_rng(77)
    n = 256
    rows = [np.sort(rng.choice(n, size=int(rng.integers(128, 224)), replace=False)) for _ in range(n)]
    rp = np.concatenate([[0], np.cumsum([r.size for r in rows])]).astype(np.int32)
    ci = np.concatenate(rows).astype(np.int32)
    per_block = 64 // dw
    assert min(r.size for r in rows) >= 8 * per_block
    X = rng.integers(-8, 9, size=(n, dim)).astype(np.float32)
    ew = rng.integers(1, 4, size=ci.size).astype(np.float32)
    G, Gw = DeviceGraph(rp, ci), DeviceGraph(rp, ci, ew)
    ref_gin = oracle.aggregate_gin(rp, ci, 1.0, X)       # (1 + eps) = 2: still integers
    ref_gcn = oracle.aggregate_gcn(rp, ci, ew, X)
    # (the workspace allows partial rows for blocks of at least 16 groups: blocks of 4 need four times the room)
    ws = gnn.alloc_workspace(n, ci.size, 4 * dim, 1)
    for rep in range(20):
        got = run_gin(G, 1.0, X, ngs=1, dw=dw, wpb=1, flags=DET, ws=ws)
        assert np.array_equal(got.view(np.uint32), ref_gin.view(np.uint32)), f"GIN, repetition {rep}"
        got = run_gcn(Gw, X, ngs=1, dw=dw, wpb=1, flags=DET, ws=ws)
        assert np.array_equal(got.view(np.uint32), ref_gcn.view(np.uint32)), f"GCN, repetition {rep}"
    # the same with a few hubs that span thousands of blocks
    star_rp, star_ci = csr_from_edges(6001, [(h, i) for h in (0, 1, 2) for i in range(3, 6001)], self_loops=True)
    Xs = rng.integers(-3, 4, size=(6001, dim)).astype(np.float32)
    Gs = DeviceGraph(star_rp, star_ci)
    ref = oracle.aggregate_gin(star_rp, star_ci, 0.0, Xs)
    wss = gnn.alloc_workspace(6001, star_ci.size, 4 * dim, 1)
    for rep in range(5):
        got = run_gin(Gs, 0.0, Xs, ngs=1, dw=dw, wpb=1, flags=DET, ws=wss)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"hubs, repetition {rep}"
