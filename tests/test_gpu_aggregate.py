"""GPU parity tests: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features
from util import csr_from_edges, random_sym_csr

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev, run_gcn, run_gin


def _graph(kind):
    if kind == "powerlaw":
        g = config_graph(2, shrink=4)  # ~4.9k nodes, hubs, self loops
        return g.rowptr, g.colidx
    if kind == "batch":
        g = config_graph(3, shrink=16)
        return g.rowptr, g.colidx
    if kind == "rmat":
        g = config_graph(5, shrink=64)  # 16k nodes, many isolated, skewed
        return g.rowptr, g.colidx
    if kind == "star":
        n = 6001
        return csr_from_edges(n, [(0, i) for i in range(1, n)], self_loops=True)
    raise ValueError(kind)


# ------------------------------------------------------------------ Sec. 4.1 / Algorithm 1 (bit-exact)
@pytest.mark.parametrize("kind", ["powerlaw", "batch", "rmat", "star"])
@pytest.mark.parametrize("ngs", [1, 2, 3, 8, 32])
def test_partition_matches_oracle(kind, ngs):
    rp, ci = _graph(kind)
    G = DeviceGraph(rp, ci)
    ws = gnn.alloc_workspace(G.n, G.nnz, 0, ngs)
    gnn.gnn_partition_build(G.n, G.nnz, G.rowptr, ngs, ws)
    node, start, end = gnn.gnn_partition_export(ws)
    onode, ostart, oend = oracle.ng_partition(rp, ngs)
    assert np.array_equal(node, onode) and np.array_equal(start, ostart) and np.array_equal(end, oend)
    _, num_ng, got_ngs = gnn.gnn_workspace_status(ws)
    assert num_ng == onode.size and got_ngs == ngs


@pytest.mark.parametrize("kind,ngs", [("powerlaw", 2), ("rmat", 4), ("star", 8)])
@pytest.mark.parametrize("dw,wpb", [(64, 1), (64, 4), (16, 4), (4, 2), (1, 1), (32, 16)])
def test_block_layout_matches_algorithm1(kind, ngs, dw, wpb):
    rp, ci = _graph(kind)
    G = DeviceGraph(rp, ci)
    ws = gnn.alloc_workspace(G.n, G.nnz, 0, ngs)
    gnn.gnn_partition_build(G.n, G.nnz, G.rowptr, ngs, ws)
    dim = 16
    slot, leader, groups_per_block = gnn.gnn_block_layout_export(ws, dim, dw, wpb)
    assert groups_per_block == wpb * (64 // dw)
    onode, _, _ = oracle.ng_partition(rp, ngs)
    oslot, _, oleader = oracle.alg1_layout(onode, groups_per_block, dim)
    assert np.array_equal(slot, oslot) and np.array_equal(leader, oleader)


# ------------------------------------------------------------------ aggregation parity
@pytest.mark.parametrize("kind", ["powerlaw", "batch", "rmat", "star"])
@pytest.mark.parametrize("dim", [16, 64, 96, 3, 22, 7, 130])
def test_gcn_parity_auto_parameters(kind, dim):
    rp, ci = _graph(kind)
    ew = oracle.gcn_norm(rp, ci)
    X = features(rp.size - 1, dim, seed=dim)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    G = DeviceGraph(rp, ci, gnn.gnn_gcn_norm(rp, ci))
    assert_parity(run_gcn(G, X), ref, ab, f"gcn {kind} dim {dim}")


@pytest.mark.parametrize("kind", ["powerlaw", "batch", "rmat", "star"])
@pytest.mark.parametrize("dim,eps", [(64, 0.0), (16, 0.5), (96, 0.0), (5, -0.25)])
def test_gin_parity_auto_parameters(kind, dim, eps):
    rp, ci = _graph(kind)
    X = features(rp.size - 1, dim, seed=100 + dim)
    ref, ab = oracle.aggregate_gin(rp, ci, eps, X, want_abs=True)
    assert_parity(run_gin(DeviceGraph(rp, ci), eps, X), ref, ab, f"gin {kind} dim {dim}")


@pytest.mark.parametrize("ngs", [1, 2, 3, 5, 8, 16, 32, 64])
@pytest.mark.parametrize("dw", [1, 2, 4, 8, 16, 32, 64])
def test_result_does_not_depend_on_ngs_dw(ngs, dw):
    rp, ci = _graph("powerlaw")
    dim = 64
    X = features(rp.size - 1, dim, seed=7)
    ew = oracle.gcn_norm(rp, ci)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    G = DeviceGraph(rp, ci, ew)
    wpb = 4 if dw >= 4 else 1
    assert_parity(run_gcn(G, X, ngs=ngs, dw=dw, wpb=wpb), ref, ab, f"ngs {ngs} dw {dw}")


@pytest.mark.parametrize("wpb", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("kind", ["rmat", "star"])
def test_result_does_not_depend_on_block_size_or_xcd_order(wpb, kind):
    rp, ci = _graph(kind)
    X = features(rp.size - 1, 64, seed=8)
    ref, ab = oracle.aggregate_gin(rp, ci, 0.0, X, want_abs=True)
    G = DeviceGraph(rp, ci)
    for ngs in (4, 32):
        for flags in (0, gnn.GNN_FLAG_XCD_RUNS, gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.GNN_FLAG_PIPELINE,
                      gnn.GNN_FLAG_ATOMIC_FLUSH | gnn.GNN_FLAG_XCD_RUNS):
            assert_parity(run_gin(G, 0.0, X, ngs=ngs, dw=16, wpb=wpb, flags=flags), ref, ab,
                          f"wpb {wpb} ngs {ngs} flags {flags}")


@pytest.mark.parametrize("kind", ["powerlaw", "rmat", "star"])
@pytest.mark.parametrize("dim,ngs", [(16, 8), (64, 32), (96, 16), (22, 4), (3, 2), (130, 8)])
def test_both_flushes_agree_with_the_oracle(kind, dim, ngs):
    rp, ci = _graph(kind)
    ew = oracle.gcn_norm(rp, ci)
    X = features(rp.size - 1, dim, seed=300 + dim)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    G = DeviceGraph(rp, ci, ew)
    for flags in (0, gnn.GNN_FLAG_ATOMIC_FLUSH):
        assert_parity(run_gcn(G, X, ngs=ngs, flags=flags), ref, ab, f"gcn {kind} dim {dim} flags {flags}")
    ref, ab = oracle.aggregate_gin(rp, ci, 0.5, X, want_abs=True)
    G2 = DeviceGraph(rp, ci)
    for flags in (0, gnn.GNN_FLAG_ATOMIC_FLUSH):
        assert_parity(run_gin(G2, 0.5, X, ngs=ngs, flags=flags), ref, ab, f"gin {kind} dim {dim} flags {flags}")


def test_unit_weights_and_integer_data_are_exact():
    # sums of small integers are exact in fp32 whatever the order: GPU == oracle bitwise
    rp, ci = _graph("rmat")
    rng = np.random.default_rng(3)
    X = rng.integers(-3, 4, size=(rp.size - 1, 32)).astype(np.float32)
    G = DeviceGraph(rp, ci)
    assert np.array_equal(run_gcn(G, X), oracle.aggregate_gcn(rp, ci, None, X))
    assert np.array_equal(run_gin(G, 1.0, X), oracle.aggregate_gin(rp, ci, 1.0, X))
    ones = np.ones((rp.size - 1, 16), dtype=np.float32)
    assert np.array_equal(run_gin(G, 0.0, ones)[:, 0], (1 + np.diff(rp)).astype(np.float32))


def test_block_level_ablation_matches_too():
    rp, ci = _graph("powerlaw")
    X = features(rp.size - 1, 16, seed=9)
    ew = oracle.gcn_norm(rp, ci)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    assert_parity(run_gcn(DeviceGraph(rp, ci, ew), X, flags=gnn.GNN_FLAG_NO_BLOCK_OPT), ref, ab, "no block opt gcn")
    ref, ab = oracle.aggregate_gin(rp, ci, 0.25, X, want_abs=True)
    assert_parity(run_gin(DeviceGraph(rp, ci), 0.25, X, flags=gnn.GNN_FLAG_NO_BLOCK_OPT), ref, ab, "no block opt gin")


def test_unaligned_rows_and_odd_dimensions_take_the_narrow_load_paths():
    rp, ci = _graph("powerlaw")
    n = rp.size - 1
    ew = oracle.gcn_norm(rp, ci)
    G = DeviceGraph(rp, ci, ew)
    for dim in (1, 2, 6, 64, 1323):
        X = features(n, dim, seed=40 + dim)
        ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
        # tensors that start 4 bytes (and 8 bytes) past a 16-byte boundary
        for shift in (1, 2):
            xbuf = torch.zeros(n * dim + 4, device="cuda")
            obuf = torch.full((n * dim + 4,), float("nan"), device="cuda")
            Xd = xbuf[shift:shift + n * dim].view(n, dim)
            Xd.copy_(dev(X))
            out = obuf[shift:shift + n * dim].view(n, dim)
            ws = gnn.alloc_workspace(G.n, G.nnz, 0, 0)
            gnn.gnn_aggregate_gcn(G.n, G.nnz, G.rowptr, G.colidx, G.ew, Xd, out, dim, 0, 0, 0, 0, ws)
            torch.cuda.synchronize()
            gnn.gnn_workspace_status(ws)
            assert_parity(out.cpu().numpy(), ref, ab, f"dim {dim} shift {shift}")
            assert torch.isnan(obuf[:shift]).all() and torch.isnan(obuf[shift + n * dim:]).all()  # nothing written outside


# ------------------------------------------------------------------ degenerate inputs
def test_empty_graph_single_node_and_isolated_nodes():
    X = features(5, 8, seed=1)
    rp = np.zeros(6, dtype=np.int32)
    ci = np.zeros(0, dtype=np.int32)
    G = DeviceGraph(rp, ci, np.zeros(0, np.float32))
    assert np.array_equal(run_gcn(G, X), np.zeros_like(X))
    assert np.array_equal(run_gin(DeviceGraph(rp, ci), 1.0, X), 2 * X)
    # one node with a self loop
    rp1 = np.array([0, 1], dtype=np.int32)
    ci1 = np.array([0], dtype=np.int32)
    x1 = features(1, 16, seed=2)
    assert np.array_equal(run_gcn(DeviceGraph(rp1, ci1, np.ones(1, np.float32)), x1), x1)
    # n = 0
    ws = gnn.alloc_workspace(0, 0)
    z = torch.zeros(1, device="cuda")
    gnn.gnn_aggregate_gin(0, 0, dev(np.zeros(1, np.int32)), dev(np.zeros(1, np.int32)), 0.0, z, z.clone(), 4, 0, 0, 0, 0, ws)
    # isolated nodes scattered between connected ones, last nodes isolated
    rp2, ci2 = csr_from_edges(70, [(0, 5), (5, 9), (9, 33), (33, 34), (2, 60)])
    X2 = features(70, 64, seed=3)
    ref, ab = oracle.aggregate_gin(rp2, ci2, 0.0, X2, want_abs=True)
    assert_parity(run_gin(DeviceGraph(rp2, ci2), 0.0, X2), ref, ab, "isolated")
    ref = oracle.aggregate_gcn(rp2, ci2, None, X2)
    got = run_gcn(DeviceGraph(rp2, ci2), X2)
    assert np.array_equal(got[np.diff(rp2) == 0], np.zeros((int((np.diff(rp2) == 0).sum()), 64), np.float32))
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)


def test_stale_workspace_and_bad_csr_are_reported():
    rp, ci = _graph("batch")
    G = DeviceGraph(rp, ci)
    X = dev(features(G.n, 16, seed=4))
    out = torch.zeros_like(X)
    ws = gnn.alloc_workspace(G.n, G.nnz, 0, 2)
    ws.zero_()
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 4, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION, ws)
    assert gnn.gnn_workspace_status(ws, check=False)[0] == -6  # GNN_ESTALE
    gnn.gnn_partition_build(G.n, G.nnz, G.rowptr, 4, ws)
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 8, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION, ws)
    assert gnn.gnn_workspace_status(ws, check=False)[0] == -6  # partition is for another ngs
    # rowptr[n] != nnz
    gnn.gnn_partition_build(G.n, G.nnz - 1, G.rowptr, 4, gnn.alloc_workspace(G.n, G.nnz, 0, 1))
    ws2 = gnn.alloc_workspace(G.n, G.nnz, 0, 1)
    gnn.gnn_partition_build(G.n, G.nnz - 1, G.rowptr, 4, ws2)
    assert gnn.gnn_workspace_status(ws2, check=False)[0] == -2  # GNN_ECSR
    with pytest.raises(gnn.GnnError):
        gnn.gnn_validate_csr_device(G.n, G.nnz - 1, G.rowptr, G.colidx)
    bad = G.colidx.clone()
    bad[5] = G.n
    with pytest.raises(gnn.GnnError):
        gnn.gnn_validate_csr_device(G.n, G.nnz, G.rowptr, bad)
    # too small / missing workspace is caught on the host
    with pytest.raises(gnn.GnnError):
        gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 4, 0, 0, 0, ws[:256])
    with pytest.raises(gnn.GnnError):
        gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, 0.0, X, out, 16, 4, 3, 0, 0, ws)  # dw not a power of two


@pytest.mark.parametrize("flags", [0, gnn.GNN_FLAG_NO_BLOCK_OPT, gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.GNN_FLAG_PIPELINE])
def test_partition_of_another_graph_of_the_same_size_is_stale(flags):
    """Renumbering keeps n and nnz (Sec. 5.1): the partition of the shuffled graph must not be accepted
    for the renumbered one."""
    g = config_graph(4, shrink=64)
    perm = gnn.gnn_reorder(g.rowptr, g.colidx, force=True)[0]
    rp2, ci2 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm)
    A, B = DeviceGraph(g.rowptr, g.colidx), DeviceGraph(rp2, ci2)
    assert (A.n, A.nnz) == (B.n, B.nnz) and not np.array_equal(g.rowptr, rp2)
    X = dev(features(A.n, 16, seed=9))
    out = torch.full_like(X, float("nan"))
    ws = gnn.alloc_workspace(A.n, A.nnz, 16, 4)
    gnn.gnn_partition_build(A.n, A.nnz, A.rowptr, 4, ws)
    gnn.gnn_aggregate_gin(B.n, B.nnz, B.rowptr, B.colidx, 0.0, X, out, 16, 4, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION | flags, ws)
    assert gnn.gnn_workspace_status(ws, check=False)[0] == -6  # GNN_ESTALE
    # built again for B, the same call computes B's aggregation
    gnn.gnn_partition_build(B.n, B.nnz, B.rowptr, 4, ws)
    gnn.gnn_aggregate_gin(B.n, B.nnz, B.rowptr, B.colidx, 0.0, X, out, 16, 4, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION | flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    ref, ab = oracle.aggregate_gin(rp2, ci2, 0.0, X.cpu().numpy(), want_abs=True)
    assert_parity(out.cpu().numpy(), ref, ab, f"rebuilt partition, flags {flags}")


def test_automatic_parameters_fit_the_scratch_memory_at_very_wide_rows():
    """Eq. 5's scratch-memory constraint in the automatic choice: no GNN_ELIMIT for wide embeddings."""
    rp, ci = _graph("powerlaw")
    n = rp.size - 1
    G = DeviceGraph(rp, ci)
    for dim in (2048, 4100, 8192):
        X = features(n, dim, seed=dim)
        ref, ab = oracle.aggregate_gin(rp, ci, 0.0, X, want_abs=True)
        assert_parity(run_gin(G, 0.0, X), ref, ab, f"automatic parameters, dim {dim}")


def test_reuse_partition_gives_identical_results():
    rp, ci = _graph("rmat")
    G = DeviceGraph(rp, ci)
    X = features(G.n, 64, seed=5)
    ws = gnn.alloc_workspace(G.n, G.nnz, 0, 8)
    a = run_gin(G, 0.0, X, ngs=8, ws=ws)
    b = run_gin(G, 0.0, X, ngs=8, flags=gnn.GNN_FLAG_REUSE_PARTITION, ws=ws)
    ref, ab = oracle.aggregate_gin(rp, ci, 0.0, X, want_abs=True)
    assert_parity(a, ref, ab, "fresh")
    assert_parity(b, ref, ab, "reused")


def test_prepared_call_equals_the_plain_call():
    rp, ci = _graph("rmat")
    ew = oracle.gcn_norm(rp, ci)
    G = DeviceGraph(rp, ci, ew)
    X = features(G.n, 24, seed=6)
    Xd = dev(X)
    ws = gnn.alloc_workspace(G.n, G.nnz, 24, 0)
    for eps, w in ((None, G.ew), (None, None), (0.25, None)):
        out = torch.full_like(Xd, float("nan"))
        call = gnn.AggregateCall(G.n, G.nnz, G.rowptr, G.colidx, w, eps, Xd, out, 24, workspace=ws)
        call()
        call()  # a prepared call can be repeated
        torch.cuda.synchronize()
        if eps is None:
            ref, ab = oracle.aggregate_gcn(rp, ci, ew if w is not None else None, X, want_abs=True)
        else:
            ref, ab = oracle.aggregate_gin(rp, ci, eps, X, want_abs=True)
        assert_parity(out.cpu().numpy(), ref, ab, f"prepared eps={eps} weighted={w is not None}")
    with pytest.raises(ValueError):
        gnn.AggregateCall(G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, Xd, out, 24, workspace=ws)


def test_renumbered_graph_gives_the_same_aggregation():
    g = config_graph(4, shrink=32)
    perm, iperm, _, did = gnn.gnn_reorder(g.rowptr, g.colidx)
    assert did
    ew = gnn.gnn_gcn_norm(g.rowptr, g.colidx)
    rp2, ci2, ew2 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm, ew)
    X = features(g.n, 96, seed=6)
    Xd, Xp = dev(X), torch.empty(g.n, 96, device="cuda")
    gnn.gnn_permute_rows(g.n, 96, dev(perm), Xd, Xp)
    assert np.array_equal(Xp.cpu().numpy(), oracle.permute_rows(X, perm))  # bit-exact row gather
    G2 = DeviceGraph(rp2, ci2, ew2)
    out_p = dev(run_gcn(G2, Xp.cpu().numpy()))
    out = torch.empty_like(out_p)
    gnn.gnn_permute_rows(g.n, 96, dev(iperm), out_p, out)
    ref, ab = oracle.aggregate_gcn(g.rowptr, g.colidx, oracle.gcn_norm(g.rowptr, g.colidx), X, want_abs=True)
    assert_parity(out.cpu().numpy(), ref, ab, "renumbered")
    back = torch.empty_like(Xd)
    gnn.gnn_permute_rows(g.n, 96, dev(iperm), Xp, back)
    assert torch.equal(back, Xd)


# ------------------------------------------------------------------ seeded random combinations
def _random_graph(rng):
    """Small graph with a random mix of empty rows, short rows and a few long rows (duplicates allowed)."""
    n = int(rng.integers(1, 700))
    deg = rng.choice([0, 1, 2, 3, 5, 9, 17, 40], size=n, p=[0.2, 0.2, 0.15, 0.15, 0.1, 0.1, 0.05, 0.05])
    for _ in range(int(rng.integers(0, 3))):
        deg[int(rng.integers(0, n))] = int(rng.integers(100, 3000))  # hubs spanning many blocks
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    ci = rng.integers(0, n, size=int(rp[-1])).astype(np.int32)
    return rp, ci


@pytest.mark.parametrize("seed", range(60))
def test_random_graphs_and_parameter_combinations(seed):
    rng = np.random.default_rng(1000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    dim = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 22, 31, 32, 64, 96, 100, 128, 200]))
    ngs = int(rng.choice([0, 1, 2, 3, 4, 7, 8, 16, 32, 64]))
    dw = int(rng.choice([0, 1, 2, 4, 8, 16, 32, 64]))
    wpb = int(rng.choice([0, 1, 2, 3, 4, 8, 16]))
    flags = int(rng.choice([0, 0, gnn.GNN_FLAG_XCD_RUNS, gnn.GNN_FLAG_PIPELINE, gnn.GNN_FLAG_NO_PIPELINE,
                            gnn.GNN_FLAG_DETERMINISTIC, gnn.GNN_FLAG_DETERMINISTIC | gnn.GNN_FLAG_XCD_RUNS,
                            gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.GNN_FLAG_ATOMIC_FLUSH | gnn.GNN_FLAG_XCD_RUNS,
                            gnn.GNN_FLAG_NO_BLOCK_OPT]))
    X = features(n, dim, seed=seed)
    what = f"seed {seed}: n {n} nnz {nnz} dim {dim} ngs {ngs} dw {dw} wpb {wpb} flags {flags}"
    print(what, flush=True)
    ws = gnn.alloc_workspace(n, nnz, dim, ngs)
    weighted = bool(rng.integers(0, 2))
    try:
        if weighted:
            ew = rng.standard_normal(nnz).astype(np.float32)
            ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
            got = run_gcn(DeviceGraph(rp, ci, ew), X, ngs=ngs, dw=dw, wpb=wpb, flags=flags, ws=ws)
        else:
            eps = float(rng.choice([0.0, 0.5, -1.0]))
            ref, ab = oracle.aggregate_gin(rp, ci, eps, X, want_abs=True)
            got = run_gin(DeviceGraph(rp, ci), eps, X, ngs=ngs, dw=dw, wpb=wpb, flags=flags, ws=ws)
    except gnn.GnnError as e:
        # a refusal must be the documented one: the scratch memory of a block above 64 KB (formula in
        # gnn.h, evaluated here on the parameters the model completes), or, with the deterministic flag,
        # blocks of fewer than 16 groups, for whose partial rows gnn_workspace_bytes leaves no room
        r_ngs, r_dw, r_wpb = gnn.gnn_decide(n, nnz, 0, dim, ngs, dw, wpb)
        T = r_wpb * (64 // r_dw)
        lds = -(-4 * (T * r_ngs + 8) * (2 if weighted else 1) // 16) * 16 + 4 * r_wpb * dim + 128 + 256 * r_wpb
        if e.code == -5:
            assert lds > 65536, f"GNN_ELIMIT although a block needs only {lds} bytes: {what}"
        else:
            assert e.code == -3 and (flags & gnn.GNN_FLAG_DETERMINISTIC) and T < 16 and lds <= 65536, f"{e.code}: {what}"
        return
    r_ngs, r_dw, r_wpb = gnn.gnn_decide(n, nnz, 0, dim, ngs, dw, wpb)
    T = r_wpb * (64 // r_dw)
    if not flags & (gnn.GNN_FLAG_NO_BLOCK_OPT | gnn.GNN_FLAG_DETERMINISTIC):
        lds = -(-4 * (T * r_ngs + 8) * (2 if weighted else 1) // 16) * 16 + 4 * r_wpb * dim + 128 + 256 * r_wpb
        assert lds <= 65536, f"accepted although a block needs {lds} bytes: {what}"
    assert_parity(got, ref, ab, what)


def test_measuring_kernels_run_and_check_their_arguments():
    X = torch.ones(1000, 64, device="cuda")
    idx = torch.randint(0, 1000, (4096,), dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, device="cuda")
    gnn.gnn_bench_stream_read(X, sink)
    gnn.gnn_bench_gather_rows(1000, 64, X, idx, sink)
    torch.cuda.synchronize()
    assert sink.item() == 0.0  # never written for finite data
    with pytest.raises(gnn.GnnError):
        gnn.gnn_bench_gather_rows(1000, 44, torch.ones(1000, 44, device="cuda"), idx, sink)  # 11 float4: no team shape
    gnn.gnn_bench_gather_rows(1000, 96, torch.ones(1000, 96, device="cuda"), idx, sink)  # 8 lanes x 3 chunks
    torch.cuda.synchronize()
