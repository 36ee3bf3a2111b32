"""GPU parity tests for the Update GEMM, whole layers, and the five configurations at full size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import BASE_SEED, config_graph, config_spec, features, glorot

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, LayerChain, assert_parity, dev, run_gcn, run_gin


@pytest.mark.parametrize("n,K,M", [(1, 1, 1), (63, 5, 3), (64, 16, 3), (1000, 500, 16), (777, 96, 16), (4097, 64, 64),
                                   (300, 16, 22), (129, 33, 70), (200, 700, 40), (50, 1323, 7), (3001, 300, 33),
                                   (65535, 256, 8), (70000, 260, 16), (5000, 512, 32), (33000, 256, 20),
                                   (70001, 64, 128), (66000, 128, 128), (66000, 130, 200), (70000, 33, 65), (4000, 256, 256),
                                   (65536, 100, 70), (65537, 8, 300)])
@pytest.mark.parametrize("relu,bias", [(False, False), (True, True)])
def test_update_gemm_parity(n, K, M, relu, bias):
    rng = np.random.default_rng(n + K + M)
    A = rng.standard_normal((n, K)).astype(np.float32)
    W = glorot(K, M, seed=K * 1000 + M)
    b = rng.standard_normal(M).astype(np.float32) if bias else None
    ref, ab = oracle.gemm_bias_act(A, W, b, relu, want_abs=True)
    out = torch.full((n, M), float("nan"), device="cuda")
    gnn.gnn_update_gemm(n, K, M, dev(A), dev(W), dev(b), relu, out)
    torch.cuda.synchronize()
    assert_parity(out.cpu().numpy(), ref, ab, f"gemm {n}x{K}x{M}")


def test_update_gemm_identity_is_exact():
    A = features(500, 64, seed=1)
    out = torch.empty(500, 64, device="cuda")
    gnn.gnn_update_gemm(500, 64, 64, dev(A), dev(np.eye(64, dtype=np.float32)), None, False, out)
    assert np.array_equal(out.cpu().numpy(), A)


@pytest.mark.parametrize("kind", ["gcn", "gin"])
@pytest.mark.parametrize("bias", [False, True])
def test_layers_with_bias_and_relu(kind, bias):
    g = config_graph(2 if kind == "gcn" else 5, shrink=4 if kind == "gcn" else 64)
    rng = np.random.default_rng(11)
    X = features(g.n, 40, seed=12)
    Ws = [glorot(40, 24, seed=13), glorot(24, 24, seed=14), glorot(24, 5, seed=15)]
    bs = [rng.standard_normal(W.shape[1]).astype(np.float32) for W in Ws] if bias else None
    if kind == "gcn":
        ew = oracle.gcn_norm(g.rowptr, g.colidx)
        LayerChain(gnn.GNN_GCN, g.rowptr, g.colidx, ew, 0.0, X, Ws, bs, name="gcn").run_to(3)
    else:
        LayerChain(gnn.GNN_GIN, g.rowptr, g.colidx, None, 0.3, X, Ws, bs, name="gin").run_to(3)


@pytest.mark.parametrize("graph", ["rmat", "batch", "powerlaw"])
@pytest.mark.parametrize("K,M,ngs,wpb", [(64, 64, 32, 4), (64, 64, 4, 4), (16, 16, 8, 4), (32, 48, 16, 4), (96, 16, 16, 4),
                                          (128, 64, 8, 4), (40, 24, 8, 2), (64, 3, 16, 4)])
@pytest.mark.parametrize("bias", [False, True])
def test_fused_gin_layer_matches_oracle_and_unfused(graph, K, M, ngs, wpb, bias):
    g = {"rmat": lambda: config_graph(5, shrink=64), "batch": lambda: config_graph(3, shrink=8),
         "powerlaw": lambda: config_graph(2, shrink=2)}[graph]()
    rng = np.random.default_rng(K + M)
    X = features(g.n, K, seed=K)
    W = glorot(K, M, seed=M)
    b = rng.standard_normal(M).astype(np.float32) if bias else None
    ref, scale = oracle.gin_layer(g.rowptr, g.colidx, 0.25, X, W, b, True, want_abs=True)
    G = DeviceGraph(g.rowptr, g.colidx)
    ws = gnn.alloc_workspace(G.n, G.nnz, max(K, M), ngs)
    outs = []
    for flags in (gnn.GNN_FLAG_FUSION, 0):
        out = torch.full((g.n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GIN, G.n, G.nnz, G.rowptr, G.colidx, None, 0.25, dev(X), K, dev(W), dev(b), M,
                              True, out, ngs, 0, wpb, flags, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs.append(out.cpu().numpy())
        assert_parity(outs[-1], ref, scale, f"gin layer {graph} {K}x{M} flags {flags}")


def _weights(cfg):
    dims = config_spec(cfg)["dims"]
    return [glorot(dims[i], dims[i + 1], BASE_SEED + cfg, stream=20 + i) for i in range(len(dims) - 1)]


def test_config1_single_gcn_aggregation_full_size():
    g = config_graph(1)
    assert (g.n, g.nnz) == (2708, 10556 + 2708)
    X = features(g.n, 16, BASE_SEED + 1)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    ref, ab = oracle.aggregate_gcn(g.rowptr, g.colidx, ew, X, want_abs=True)
    G = DeviceGraph(g.rowptr, g.colidx, gnn.gnn_gcn_norm(g.rowptr, g.colidx))
    assert_parity(run_gcn(G, X), ref, ab, "config 1")


def test_config2_two_layer_gcn_full_size():
    g = config_graph(2)
    assert (g.n, g.nnz) == (19717, 88648 + 19717)
    X = features(g.n, 500, BASE_SEED + 2)
    ew = gnn.gnn_gcn_norm(g.rowptr, g.colidx)
    assert ew.tobytes() == oracle.gcn_norm(g.rowptr, g.colidx).tobytes()
    LayerChain(gnn.GNN_GCN, g.rowptr, g.colidx, ew, 0.0, X, _weights(2), name="config 2").run_to(2)


def test_config3_five_layer_gin_full_size():
    g = config_graph(3)
    X = features(g.n, 64, BASE_SEED + 3)
    LayerChain(gnn.GNN_GIN, g.rowptr, g.colidx, None, 0.0, X, _weights(3), name="config 3").run_to(5)


# Configurations 4 and 5 take the oracle several seconds per layer: one test per layer, state kept
# between them (a layer's test first runs whatever earlier layers are still missing).
_chains = {}


def _config4_chain(renumber):
    key = ("cfg4", renumber)
    if key not in _chains:
        g = config_graph(4)
        assert (g.n, g.nnz) == (410236, 4878874 + 410236)
        rp, ci = g.rowptr, g.colidx
        X = features(g.n, 96, BASE_SEED + 4)
        ew = gnn.gnn_gcn_norm(rp, ci)
        if renumber:
            perm, iperm, _, did = gnn.gnn_reorder(rp, ci)
            assert did
            assert np.array_equal(perm, oracle.reorder(rp, ci)[0])  # bit-exact renumbering at full size
            rp, ci, ew = gnn.gnn_apply_perm_csr(rp, ci, perm, ew)
            orp, oci, oew = oracle.apply_perm_csr(g.rowptr, g.colidx, perm, oracle.gcn_norm(g.rowptr, g.colidx))
            assert rp.tobytes() == orp.tobytes() and ci.tobytes() == oci.tobytes() and ew.tobytes() == oew.tobytes()
            Xd = torch.empty(g.n, 96, device="cuda")
            gnn.gnn_permute_rows(g.n, 96, dev(perm), dev(X), Xd)
            assert np.array_equal(Xd.cpu().numpy(), oracle.permute_rows(X, perm))
            X = Xd.cpu().numpy()
        _chains[key] = (LayerChain(gnn.GNN_GCN, rp, ci, ew, 0.0, X, _weights(4), name=f"config 4 renumber={renumber}"),
                        rp, ci, ew, X)
    return _chains[key]


@pytest.mark.parametrize("renumber", [False, True])
def test_config4_aggregation_dim96_full_size(renumber):
    chain, rp, ci, ew, X = _config4_chain(renumber)
    ref, ab = oracle.aggregate_gcn(rp, ci, ew, X, want_abs=True)
    assert_parity(run_gcn(chain.G, X), ref, ab, f"config 4 aggregation renumber={renumber}")


@pytest.mark.parametrize("renumber", [False, True])
@pytest.mark.parametrize("layer", [1, 2])
def test_config4_two_layer_gcn_full_size(renumber, layer):
    _config4_chain(renumber)[0].run_to(layer)


def _config5_chain(ngs):
    key = ("cfg5", ngs)
    if key not in _chains:
        g = config_graph(5)
        assert g.n == 1 << 20
        X = features(g.n, 64, BASE_SEED + 5)
        _chains[key] = LayerChain(gnn.GNN_GIN, g.rowptr, g.colidx, None, 0.0, X, _weights(5), ngs=ngs,
                                  name=f"config 5 ngs={ngs}")
    return _chains[key]


@pytest.mark.parametrize("layer", [1, 2, 3, 4, 5])
def test_config5_five_layer_gin_full_size(layer):
    _config5_chain(0).run_to(layer)


@pytest.mark.parametrize("ngs", [2, 4, 8, 16, 32])
def test_config5_aggregation_for_every_group_size_of_the_sweep(ngs):
    chain = _config5_chain(0)
    g = config_graph(5)
    X = features(g.n, 64, BASE_SEED + 5)
    key = ("cfg5", "agg_ref")
    if key not in _chains:
        _chains[key] = oracle.aggregate_gin(g.rowptr, g.colidx, 0.0, X, want_abs=True)
    ref, ab = _chains[key]
    assert_parity(run_gin(chain.G, 0.0, X, ngs=ngs), ref, ab, f"config 5 aggregation ngs {ngs}")


def test_config5_renumbered_at_full_size_gives_the_same_aggregation():
    """Sec. 5.1: renumbering must not change the result.  The largest graph at full size: the library's
    permutation and relabelled CSR equal the oracle's byte for byte, and the GIN aggregation of the
    renumbered graph, rows moved back, equals the oracle's aggregation of the original graph."""
    g = config_graph(5)
    X = features(g.n, 64, BASE_SEED + 5)
    perm, iperm, _, did = gnn.gnn_reorder(g.rowptr, g.colidx)
    assert did  # Eq. 4 of the scrambled ids is far above the rule's threshold
    operm, oiperm = oracle.reorder(g.rowptr, g.colidx)
    assert perm.tobytes() == operm.tobytes() and iperm.tobytes() == oiperm.tobytes()
    rp2, ci2 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm)
    orp, oci = oracle.apply_perm_csr(g.rowptr, g.colidx, operm)
    assert rp2.tobytes() == orp.tobytes() and ci2.tobytes() == oci.tobytes()
    G2 = DeviceGraph(rp2, ci2)
    Xp = torch.empty(g.n, 64, device="cuda")
    gnn.gnn_permute_rows(g.n, 64, dev(perm), dev(X), Xp)
    assert np.array_equal(Xp.cpu().numpy(), oracle.permute_rows(X, perm))
    out2 = torch.full((g.n, 64), float("nan"), device="cuda")
    ws = gnn.alloc_workspace(G2.n, G2.nnz, 64, 0)
    gnn.gnn_aggregate_gin(G2.n, G2.nnz, G2.rowptr, G2.colidx, 0.0, Xp, out2, 64, 0, 0, 0, 0, ws)
    back = torch.empty_like(out2)
    gnn.gnn_permute_rows(g.n, 64, dev(iperm), out2, back)  # row perm[i] of the renumbered result is node i
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    key = ("cfg5", "agg_ref")
    if key not in _chains:
        _chains[key] = oracle.aggregate_gin(g.rowptr, g.colidx, 0.0, X, want_abs=True)
    ref, ab = _chains[key]
    assert_parity(back.cpu().numpy(), ref, ab, "config 5 renumbered, rows moved back")


# ------------------------------------------------------------------ whole model in one call
@pytest.mark.parametrize("cfg,shrink", [(2, 4), (3, 8), (4, 32)])
def test_model_forward_equals_the_layer_by_layer_chain_and_the_oracle(cfg, shrink):
    from gnn_synth import config_spec
    from util import parity_errors
    from gpu_util import TOL, run_model
    spec = config_spec(cfg)
    g = config_graph(cfg, shrink=shrink)
    dims = list(spec["dims"])
    kind = gnn.GNN_GIN if spec["kind"] == "gin" else gnn.GNN_GCN
    X = features(g.n, dims[0], seed=cfg)
    Ws = [glorot(dims[i], dims[i + 1], seed=10 * cfg + i) for i in range(len(dims) - 1)]
    bs = [features(1, dims[i + 1], seed=50 + i)[0] * 0.1 if i % 2 == 0 else None for i in range(len(dims) - 1)]
    ew = oracle.gcn_norm(g.rowptr, g.colidx) if kind == gnn.GNN_GCN else None
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    ws = torch.empty(gnn.gnn_model_workspace_bytes(G.n, G.nnz, dims, 0), dtype=torch.uint8, device="cuda")
    out = torch.full((G.n, dims[-1]), float("nan"), device="cuda")
    Wd = [dev(W) for W in Ws]
    bd = [None if b is None else dev(b) for b in bs]
    model = gnn.ModelCall(kind, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), dims, Wd, bd, out, workspace=ws)
    model()
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    first = out.cpu().numpy().copy()
    # same kernels in the same order as the chain of gnn_layer_forward calls: identical bits
    chain = run_model(kind, G, 0.0, X, Ws, bs)
    assert np.array_equal(first.view(np.uint32), chain.view(np.uint32))
    ref = (oracle.gcn_model(g.rowptr, g.colidx, ew, X, Ws, bs) if kind == gnn.GNN_GCN
           else oracle.gin_model(g.rowptr, g.colidx, 0.0, X, Ws, bs))
    normwise, _ = parity_errors(first, ref, None)
    assert normwise <= TOL, normwise
    # a second call reusing the partition gives the same bits
    out.fill_(float("nan"))
    model(flags=gnn.GNN_FLAG_REUSE_PARTITION)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), first.view(np.uint32))
    # too small a workspace is refused on the host
    with pytest.raises(gnn.GnnError):
        gnn.gnn_model_forward(kind, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), dims, Wd, bd, out, workspace=ws[:4096])


def test_widening_gcn_layer_aggregates_first_unless_told_otherwise():
    g = config_graph(4, shrink=16)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    X = features(g.n, 16, seed=91)
    W = glorot(16, 22, seed=92)
    b = features(1, 22, seed=93)[0] * 0.1
    ref, scale = oracle.gcn_layer(g.rowptr, g.colidx, ew, X, W, b, True, want_abs=True)
    ws = gnn.alloc_workspace(G.n, G.nnz, 22, 0)
    outs = {}
    for flags in (0, gnn.GNN_FLAG_GCN_UPDATE_FIRST):
        out = torch.full((G.n, 22), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GCN, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 16, dev(W), dev(b), 22, True,
                              out, 0, 0, 0, flags, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs[flags] = out.cpu().numpy()
        # A_hat (X W) = (A_hat X) W: the same oracle value, the same error scale
        assert_parity(outs[flags], ref, scale, f"gcn layer 16->22 flags {flags}")
    # a narrowing layer ignores the flag: identical bits
    W2 = glorot(22, 16, seed=94)
    X2 = features(g.n, 22, seed=95)
    res = []
    for flags in (0, gnn.GNN_FLAG_GCN_UPDATE_FIRST):
        out = torch.full((G.n, 16), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GCN, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X2), 22, dev(W2), None, 16, False,
                              out, 0, 0, 0, flags, ws)
        torch.cuda.synchronize()
        res.append(out.cpu().numpy())
    assert np.array_equal(res[0].view(np.uint32), res[1].view(np.uint32))


def test_fusion_is_automatic_for_short_rows_and_can_be_switched_off():
    """A GIN layer on a batch of small graphs (mean row < 8) runs fused by itself; GNN_FLAG_NO_FUSION
    gives the two separate kernels.  Both match the oracle; rows complete inside one block (all of
    them here) see the same arithmetic either way up to the order of the MFMA steps."""
    g = config_graph(3, shrink=4)
    K, M = 64, 64
    X = features(g.n, K, seed=301)
    W = glorot(K, M, seed=302)
    b = features(1, M, seed=303)[0] * 0.1
    ref, scale = oracle.gin_layer(g.rowptr, g.colidx, 0.0, X, W, b, True, want_abs=True)
    G = DeviceGraph(g.rowptr, g.colidx)
    ws = gnn.alloc_workspace(G.n, G.nnz, 64, 0)
    outs = []
    for flags in (0, gnn.GNN_FLAG_NO_FUSION, gnn.GNN_FLAG_FUSION, gnn.GNN_FLAG_DETERMINISTIC):
        out = torch.full((G.n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GIN, G.n, G.nnz, G.rowptr, G.colidx, None, 0.0, dev(X), K, dev(W), dev(b), M, True, out,
                              0, 0, 0, flags, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs.append(out.cpu().numpy())
        assert_parity(outs[-1], ref, scale, f"gin layer flags {flags}")
        fused = gnn.gnn_bench_last_aggregation().startswith("k_gin_layer_fused")
        assert fused == (flags != gnn.GNN_FLAG_NO_FUSION), (flags, gnn.gnn_bench_last_aggregation())
    assert np.array_equal(outs[0].view(np.uint32), outs[2].view(np.uint32))  # automatic == requested fusion
    assert np.array_equal(outs[0].view(np.uint32), outs[3].view(np.uint32))  # the fused kernel is deterministic


@pytest.mark.parametrize("K,dw,M", [(64, 8, 64), (64, 16, 64), (32, 8, 48), (32, 4, 16), (16, 4, 22)])
@pytest.mark.parametrize("ngs", [1, 3, 16])
def test_fused_wave_tiles_with_nodes_that_span_rounds_waves_and_tiles(K, dw, M, ngs):
    """The wave-tile form of the fused GIN layer (a wave owns 16 groups, rows of the tile per target node,
    ordered flush of the transformed partial rows in units of wave tiles) on a graph with hubs and with
    groups so small that nodes continue from one round, wave and tile into the next.  X, W and b hold small
    integers, so every sum is exact in fp32 whatever its order: the result must equal the oracle bit for
    bit -- a partial row that was stale, counted twice or left out could not hide in rounding -- and so must
    a second run."""
    g = config_graph(5, shrink=64)
    rng = np.random.default_rng(K * 1000 + M * 10 + ngs)
    X = rng.integers(-3, 4, size=(g.n, K)).astype(np.float32)
    W = rng.integers(-2, 3, size=(K, M)).astype(np.float32)
    b = rng.integers(-4, 5, size=M).astype(np.float32)
    ref = oracle.gin_layer(g.rowptr, g.colidx, 1.0, X, W, b, True)
    G = DeviceGraph(g.rowptr, g.colidx)
    ws = gnn.alloc_workspace(G.n, G.nnz, max(K, M), ngs)
    outs = []
    for _ in range(2):
        out = torch.full((g.n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GIN, G.n, G.nnz, G.rowptr, G.colidx, None, 1.0, dev(X), K, dev(W), dev(b), M, True, out,
                              ngs, dw, 0, gnn.GNN_FLAG_FUSION, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        assert gnn.gnn_bench_last_aggregation().startswith("k_gin_layer_fused_w"), gnn.gnn_bench_last_aggregation()
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], ref.astype(np.float32)), np.abs(outs[0] - ref).max()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


@pytest.mark.parametrize("K,M,ngs", [(16, 22, 32), (16, 22, 5), (32, 48, 16), (16, 64, 8), (64, 70, 32)])
def test_fused_gcn_layer_that_widens(K, M, ngs):
    """A GCN layer whose output is wider than its input aggregates first; with GNN_FLAG_FUSION the Update is
    fused into that aggregation (wave-tile form with the edge weights beside the indices, no own-row term)
    where the shape is covered.  Oracle values with the Eq. 2 weights; then integer-valued data and weights,
    for which every sum is exact: bit-equal to the oracle and from run to run."""
    g = config_graph(4, shrink=16)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    X = features(g.n, K, seed=K + M)
    W = glorot(K, M, seed=M)
    b = features(1, M, seed=ngs)[0] * 0.1
    ref, scale = oracle.gcn_layer(g.rowptr, g.colidx, ew, X, W, b, True, want_abs=True)
    ws = gnn.alloc_workspace(G.n, G.nnz, max(K, M), ngs)
    out = torch.full((g.n, M), float("nan"), device="cuda")
    gnn.gnn_layer_forward(gnn.GNN_GCN, G.n, G.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), K, dev(W), dev(b), M, True, out,
                          ngs, 0, 0, gnn.GNN_FLAG_FUSION, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    name = gnn.gnn_bench_last_aggregation()
    covered = M <= 64
    assert name.startswith("k_gin_layer_fused_w") == covered, name
    assert_parity(out.cpu().numpy(), ref, scale, f"fused gcn layer {K}->{M} ngs {ngs}")

    rng = np.random.default_rng(K * M + ngs)
    Xi = rng.integers(-3, 4, size=(g.n, K)).astype(np.float32)
    Wi = rng.integers(-2, 3, size=(K, M)).astype(np.float32)
    bi = rng.integers(-4, 5, size=M).astype(np.float32)
    ewi = rng.integers(1, 3, size=g.nnz).astype(np.float32)
    refi = oracle.gcn_layer(g.rowptr, g.colidx, ewi, Xi, Wi, bi, True)
    Gi = DeviceGraph(g.rowptr, g.colidx, ewi)
    outs = []
    for _ in range(2):
        out = torch.full((g.n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GCN, Gi.n, Gi.nnz, Gi.rowptr, Gi.colidx, Gi.ew, 0.0, dev(Xi), K, dev(Wi), dev(bi), M, True,
                              out, ngs, 0, 0, gnn.GNN_FLAG_FUSION, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], refi.astype(np.float32)), np.abs(outs[0] - refi).max()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


def _random_graph(rng):
    """Degrees from one of several shapes (regular, short rows, a few hubs, many empty rows); duplicate and
    self entries allowed."""
    n = int(rng.choice([1, 17, 300, 5000, 40000]))
    kind = int(rng.integers(0, 4))
    if kind == 0:
        deg = np.full(n, int(rng.integers(1, 9)))
    elif kind == 1:
        deg = rng.integers(0, 11, size=n)
    elif kind == 2:
        deg = rng.integers(0, 4, size=n)
        deg[rng.integers(0, n, size=max(1, n // 200))] = rng.integers(200, 3000)
    else:
        deg = np.where(rng.random(n) < 0.7, 0, rng.integers(1, 40, size=n))
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    ci = rng.integers(0, n, size=int(rp[-1])).astype(np.int32)
    return rp, ci


@pytest.mark.parametrize("seed", range(40))
def test_fused_layers_on_random_graphs_and_shapes(seed):
    """Random graphs, widths, group sizes, team widths, bias / activation, GIN and widening GCN layers with
    GNN_FLAG_FUSION: whichever form of the fused layer the library picks (or none, where no form covers the
    shape) must match the oracle, and a second run must repeat the first bit for bit."""
    rng = np.random.default_rng(7000 + seed)
    rp, ci = _random_graph(rng)
    n, nnz = rp.size - 1, ci.size
    K = int(rng.choice([16, 32, 64, 64, 24, 128]))
    M = int(rng.choice([1, 3, 16, 22, 48, 64, 64, 70]))
    ngs = int(rng.choice([0, 1, 2, 5, 8, 16, 32, 64]))
    dw = int(rng.choice([0, 0, 4, 8, 16]))
    gcn = bool(rng.integers(0, 2)) and M > K
    relu = bool(rng.integers(0, 2))
    X = features(n, K, seed=seed)
    W = glorot(K, M, seed=seed + 1)
    b = features(1, M, seed=seed + 2)[0] if rng.integers(0, 2) else None
    what = f"seed {seed}: n {n} nnz {nnz} {'gcn' if gcn else 'gin'} {K}->{M} ngs {ngs} dw {dw} relu {relu} bias {b is not None}"
    print(what, flush=True)
    if gcn:
        ew = rng.standard_normal(nnz).astype(np.float32)
        ref, scale = oracle.gcn_layer(rp, ci, ew, X, W, b, relu, want_abs=True)
        G, kind, eps = DeviceGraph(rp, ci, ew), gnn.GNN_GCN, 0.0
    else:
        eps = float(rng.choice([0.0, 0.5, -1.0]))
        ref, scale = oracle.gin_layer(rp, ci, eps, X, W, b, relu, want_abs=True)
        G, kind = DeviceGraph(rp, ci), gnn.GNN_GIN
    ws = gnn.alloc_workspace(n, nnz, max(K, M), ngs)
    outs = []
    for _ in range(2):
        out = torch.full((n, M), float("nan"), device="cuda")
        gnn.gnn_layer_forward(kind, n, nnz, G.rowptr, G.colidx, G.ew if gcn else None, eps, dev(X), K, dev(W), dev(b), M, relu,
                              out, ngs, dw, 0, gnn.GNN_FLAG_FUSION, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        outs.append(out.cpu().numpy())
    print("   ", gnn.gnn_bench_last_aggregation(), flush=True)
    assert_parity(outs[0], ref, scale, what)
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32)), what


def test_fused_layer_takes_the_block_tile_form_where_the_wave_tile_form_does_not_apply():
    # rows of 96 floats, and groups of more entries than a team keeps in registers
    g = config_graph(3, shrink=8)
    G = DeviceGraph(g.rowptr, g.colidx)
    for K, ngs in ((96, 16), (64, 64)):
        X = features(g.n, K, seed=K)
        W = glorot(K, 32, seed=ngs)
        ref, scale = oracle.gin_layer(g.rowptr, g.colidx, 0.0, X, W, None, False, want_abs=True)
        ws = gnn.alloc_workspace(G.n, G.nnz, K, ngs)
        out = torch.full((g.n, 32), float("nan"), device="cuda")
        gnn.gnn_layer_forward(gnn.GNN_GIN, G.n, G.nnz, G.rowptr, G.colidx, None, 0.0, dev(X), K, dev(W), None, 32, False, out,
                              ngs, 0, 0, gnn.GNN_FLAG_FUSION, ws)
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(ws)
        name = gnn.gnn_bench_last_aggregation()
        assert name.startswith("k_gin_layer_fused<"), name
        assert_parity(out.cpu().numpy(), ref, scale, f"block-tile fused layer K {K} ngs {ngs}")


@pytest.mark.parametrize("out_dim", [1, 2, 3, 5, 6, 7, 22, 33, 70])
@pytest.mark.parametrize("flags", [0, gnn.GNN_FLAG_ATOMIC_FLUSH, gnn.GNN_FLAG_DETERMINISTIC, gnn.GNN_FLAG_XCD_RUNS,
                                   gnn.GNN_FLAG_NO_BLOCK_OPT])
def test_gcn_layer_with_a_width_that_is_not_a_multiple_of_four(out_dim, flags):
    # rows of such a width are not 16-byte aligned: the narrow load and store paths; nothing may be
    # written past the end of `out`
    g = config_graph(4, shrink=32)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    rng = np.random.default_rng(out_dim)
    X = features(g.n, 24, seed=3)
    W = glorot(24, out_dim, seed=out_dim)
    b = rng.standard_normal(out_dim).astype(np.float32)
    ref, ab = oracle.gcn_layer(g.rowptr, g.colidx, ew, X, W, b, True, want_abs=True)
    guard = 64
    buf = torch.full((g.n * out_dim + guard,), float("nan"), device="cuda")
    out = buf[: g.n * out_dim].view(g.n, out_dim)
    ws = gnn.alloc_workspace(g.n, g.nnz, max(24, out_dim), 0)
    gnn.gnn_layer_forward(gnn.GNN_GCN, g.n, g.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 24, dev(W), dev(b), out_dim, True,
                          out, 0, 0, 0, flags, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    assert_parity(out.cpu().numpy(), ref, ab, f"gcn layer 24->{out_dim} flags={flags}")
    assert torch.isnan(buf[g.n * out_dim:]).all()


def test_gcn_layer_in_a_workspace_without_room_for_partial_rows():
    g = config_graph(4, shrink=32)
    ew = oracle.gcn_norm(g.rowptr, g.colidx)
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    X = features(g.n, 16, seed=4)
    W = glorot(16, 22, seed=5)
    ref, ab = oracle.gcn_layer(g.rowptr, g.colidx, ew, X, W, None, False, want_abs=True)
    out = torch.full((g.n, 22), float("nan"), device="cuda")
    full = gnn.alloc_workspace(g.n, g.nnz, 22, 16)
    # keep the intermediate (Update first: 22 floats per node), drop the partial rows: rows that span blocks
    # are finished with atomics
    tight = full[: gnn.gnn_workspace_bytes(g.n, g.nnz, 0, 16) + ((g.n * 22 * 4 + 255) // 256) * 256]
    assert tight.numel() < full.numel()
    with pytest.raises(gnn.GnnError):
        gnn.gnn_layer_forward(gnn.GNN_GCN, g.n, g.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 16, dev(W), None, 22, False,
                              out, 16, 0, 0, gnn.GNN_FLAG_DETERMINISTIC | gnn.GNN_FLAG_GCN_UPDATE_FIRST, tight)
    gnn.gnn_layer_forward(gnn.GNN_GCN, g.n, g.nnz, G.rowptr, G.colidx, G.ew, 0.0, dev(X), 16, dev(W), None, 22, False, out,
                          16, 0, 0, gnn.GNN_FLAG_GCN_UPDATE_FIRST, tight)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(tight)
    assert_parity(out.cpu().numpy(), ref, ab, "gcn layer 16->22, tight workspace")


@pytest.mark.parametrize("kind", ["gcn", "gin"])
def test_model_forward_captured_in_a_hip_graph_replays_like_the_eager_call(kind):
    # the device entry points only enqueue kernels (no memset nodes, no synchronisation), so a caller can
    # capture them; every replay, with eager work and new inputs in between, must equal the eager call
    g = config_graph(2, shrink=4) if kind == "gcn" else config_graph(3, shrink=8)
    dims = [24, 16, 5] if kind == "gcn" else [32, 32, 32]
    ew = oracle.gcn_norm(g.rowptr, g.colidx) if kind == "gcn" else None
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    Ws = [dev(glorot(dims[i], dims[i + 1], seed=40 + i)) for i in range(len(dims) - 1)]
    X = dev(features(g.n, dims[0], seed=50))
    out = torch.empty(g.n, dims[-1], device="cuda")
    mws = torch.empty(gnn.gnn_model_workspace_bytes(g.n, g.nnz, dims, 0), dtype=torch.uint8, device="cuda")
    ngs, _, _ = gnn.gnn_decide(g.n, g.nnz, 0, dims[0])
    gnn.gnn_partition_build(g.n, g.nnz, G.rowptr, ngs, mws)
    call = gnn.ModelCall(gnn.GNN_GCN if kind == "gcn" else gnn.GNN_GIN, g.n, g.nnz, G.rowptr, G.colidx, G.ew, 0.1, X, dims,
                         Ws, None, out, ngs, 0, 0, gnn.GNN_FLAG_REUSE_PARTITION, mws)
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        call()
    for k in range(3):
        X.copy_(dev(features(g.n, dims[0], seed=60 + k)))  # eager work between the replays
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        replayed = out.clone()
        out.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        assert torch.equal(out, replayed), f"replay {k} differs from the eager call"
        assert not torch.isnan(replayed).any()
    gnn.gnn_workspace_status(mws)


@pytest.mark.parametrize("seed", range(24))
def test_update_gemm_random_shapes(seed):
    # the shape decides among four kernels (streaming, resident W, W travelling with A, K split over
    # the waves) and their 4- / 16-byte load forms: draw shapes across all of them
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 7, 100, 1000, 5000, 20000, 40000, 70000]) * rng.uniform(0.5, 1.0)) + 1
    K = int(rng.choice([3, 16, 32, 33, 64, 100, 128, 255, 256, 500, 1433]))
    M = int(rng.choice([1, 3, 7, 16, 22, 32, 47, 64, 65, 100]))
    if n * K > 40_000_000:
        n = 40_000_000 // K
    A = rng.standard_normal((n, K)).astype(np.float32)
    W = glorot(K, M, seed=seed)
    b = rng.standard_normal(M).astype(np.float32) if seed % 2 else None
    relu = seed % 3 == 0
    ref, ab = oracle.gemm_bias_act(A, W, b, relu, want_abs=True)
    out = torch.full((n, M), float("nan"), device="cuda")
    gnn.gnn_update_gemm(n, K, M, dev(A), dev(W), dev(b), relu, out)
    torch.cuda.synchronize()
    assert_parity(out.cpu().numpy(), ref, ab, f"gemm {n}x{K}x{M} seed {seed}")
