"""gnn_aggregate_gin_static (the entry point that allocates nothing: its partition, counters and partial
rows live in a fixed device array inside the library) against gnn_aggregate_gin with a caller's
workspace, through the C ABI: two calls in a row, the second on a smaller input, then the limit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev


def _both(g, dim, seed, flags=0, ngs=0):
    G = DeviceGraph(g.rowptr, g.colidx)
    X = features(g.n, dim, seed=seed)
    Xd = dev(X)
    ref_out = torch.full((g.n, dim), float("nan"), device="cuda")
    ws = gnn.alloc_workspace(G.n, G.nnz, dim, ngs)
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.25, Xd, ref_out, dim, ngs, 0, 0, flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    out = torch.full((g.n, dim), float("nan"), device="cuda")
    before = torch.cuda.memory_allocated()
    scratch = gnn.gnn_aggregate_gin_static(G.n, G.nnz, G.rowptr, G.colidx, 0.25, Xd, out, dim, ngs, 0, 0, flags)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert scratch != 0
    status, num_ng, _ = gnn.gnn_workspace_status(scratch)
    assert status == 0 and num_ng == gnn.gnn_workspace_status(ws)[1]
    return G, Xd, X, out, ref_out, scratch


def test_static_scratch_entry_point_matches_the_workspace_entry_point_twice_in_a_row():
    big = config_graph(5, shrink=8)      # 131,072 nodes, skewed, hubs that span many blocks, empty rows
    small = config_graph(2, shrink=2)    # 9,858 nodes
    for g, dim, seed in ((big, 64, 11), (small, 22, 12)):
        G, Xd, X, out, ref_out, scratch = _both(g, dim, seed)
        print(f"static scratch: n {g.n} nnz {g.nnz} dim {dim}", flush=True)
        got, want = out.cpu().numpy(), ref_out.cpu().numpy()
        # same kernels, same parameters, ordered flush on both sides: the same bits
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        ref, ab = oracle.aggregate_gin(g.rowptr, g.colidx, 0.25, X, want_abs=True)
        assert_parity(got, ref, ab, f"static scratch n {g.n}")
    # the array keeps the last call's partition: reuse is honoured for the same graph ...
    out2 = torch.full_like(out, float("nan"))
    gnn.gnn_aggregate_gin_static(G.n, G.nnz, G.rowptr, G.colidx, 0.25, Xd, out2, dim, 0, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION)
    torch.cuda.synchronize()
    assert gnn.gnn_workspace_status(scratch)[0] == 0
    assert torch.equal(out2, out)
    # ... and refused for another one
    Gb = DeviceGraph(big.rowptr, big.colidx)
    outb = torch.zeros(big.n, 16, device="cuda")
    gnn.gnn_aggregate_gin_static(Gb.n, Gb.nnz, Gb.rowptr, Gb.colidx, 0.0, dev(features(big.n, 16, seed=1)), outb, 16, 0, 0, 0,
                                 gnn.GNN_FLAG_REUSE_PARTITION)
    assert gnn.gnn_workspace_status(scratch, check=False)[0] == -6  # GNN_ESTALE


def test_static_scratch_entry_point_with_the_atomic_flush_and_small_groups():
    g = config_graph(4, shrink=32)
    for flags, ngs in ((gnn.GNN_FLAG_ATOMIC_FLUSH, 0), (0, 4), (gnn.GNN_FLAG_DETERMINISTIC, 16)):
        G, Xd, X, out, ref_out, _ = _both(g, 32, 13, flags=flags, ngs=ngs)
        ref, ab = oracle.aggregate_gin(g.rowptr, g.colidx, 0.25, X, want_abs=True)
        assert_parity(out.cpu().numpy(), ref, ab, f"static scratch flags {flags} ngs {ngs}")
        assert_parity(out.cpu().numpy(), ref_out.cpu().numpy(), ab, f"static scratch against the workspace call, flags {flags}")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    n, nnz = 40_000_000, 200_000_000  # the partition alone would need more than 128 MiB
    assert gnn.gnn_workspace_bytes(n, nnz, 64, 0) > 128 << 20
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    f = torch.zeros(8, device="cuda")
    with pytest.raises(gnn.GnnError) as e:
        gnn.gnn_aggregate_gin_static(n, nnz, t, t, 0.0, f, f.clone(), 64)  # refused before anything is read
    assert e.value.code == -5
    with pytest.raises(gnn.GnnError):
        gnn.gnn_aggregate_gin_static(8, 0, t, t, 0.0, f, f, 1)  # in and out alias
