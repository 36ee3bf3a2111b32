"""Tensors with more than 2^31 elements: every row offset must be computed in 64 bits.

The feature matrix (8.5 M x 256 floats, 8.7 GB) lives only on the GPU; the rows the checks need are
copied to the host and handed to the oracle as a small graph with compacted ids."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, assert_parity, dev

N, DIM = 8_500_000, 256  # N * DIM = 2.176e9 > 2^31


def _sparse_rows_graph(rng, n, rows, max_deg):
    """CSR with entries only in `rows` (sorted node ids): 1..max_deg random neighbours each."""
    deg = np.zeros(n, dtype=np.int64)
    deg[rows] = rng.integers(1, max_deg + 1, size=rows.size)
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rp[1:])
    ci = rng.integers(0, n, size=int(rp[-1])).astype(np.int32)
    ci[-1] = n - 1  # the very last row of X is read too
    return rp.astype(np.int32), ci


def test_aggregation_with_more_than_2_31_elements():
    free, _ = torch.cuda.mem_get_info()
    if free < 40e9:
        pytest.skip("needs about 20 GB of device memory")
    rng = np.random.default_rng(2031)
    gen = torch.Generator(device="cuda").manual_seed(2031)
    X = torch.randn(N, DIM, device="cuda", generator=gen)
    rows = np.unique(np.concatenate([rng.integers(0, N, size=20000), np.arange(N - 64, N), np.arange(0, 64)]))
    rp, ci = _sparse_rows_graph(rng, N, rows, 40)
    G = DeviceGraph(rp, ci)
    out = torch.full((N, DIM), float("nan"), device="cuda")
    ws = gnn.alloc_workspace(G.n, G.nnz, 0, 0)
    eps = 0.5
    print(f"large aggregation: n {N} dim {DIM} nnz {G.nnz}", flush=True)
    gnn.gnn_aggregate_gin(G.n, G.nnz, G.rowptr, G.colidx, eps, X, out, DIM, 0, 0, 0, 0, ws)
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)

    # oracle on the compacted graph: the sampled rows and everything they reference
    used = np.unique(np.concatenate([rows, ci]))
    remap = np.full(N, -1, dtype=np.int64)
    remap[used] = np.arange(used.size)
    deg = np.diff(rp.astype(np.int64))
    crp = np.zeros(used.size + 1, dtype=np.int64)
    np.cumsum(deg[used], out=crp[1:])
    cci = remap[ci.astype(np.int64)].astype(np.int32)  # entries of `rows` in order; other used nodes have none
    Xs = X[torch.from_numpy(used).cuda()].cpu().numpy()
    ref, ab = oracle.aggregate_gin(crp.astype(np.int32), cci, eps, Xs, want_abs=True)
    got = out[torch.from_numpy(used).cuda()].cpu().numpy()
    assert_parity(got, ref, ab, "2^31+ elements, sampled rows and their neighbours")
    # rows without entries: (1 + eps) * x exactly, checked on a large random sample
    sample = torch.from_numpy(rng.integers(0, N, size=200000)).cuda()
    empty = sample[torch.from_numpy(deg[sample.cpu().numpy()] == 0).cuda()]
    assert torch.equal(out[empty], (1.0 + eps) * X[empty])
    assert not torch.isnan(out[-1]).any() and not torch.isnan(out).any()


def test_update_gemm_with_more_than_2_31_elements():
    free, _ = torch.cuda.mem_get_info()
    if free < 20e9:
        pytest.skip("needs about 10 GB of device memory")
    rng = np.random.default_rng(2032)
    gen = torch.Generator(device="cuda").manual_seed(2032)
    A = torch.randn(N, DIM, device="cuda", generator=gen)
    M = 16
    W = (rng.standard_normal((DIM, M)) / 16).astype(np.float32)
    b = rng.standard_normal(M).astype(np.float32)
    out = torch.full((N, M), float("nan"), device="cuda")
    print(f"large GEMM: n {N} K {DIM} M {M}", flush=True)
    gnn.gnn_update_gemm(N, DIM, M, A, dev(W), dev(b), True, out)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.integers(0, N, size=4096), np.arange(N - 70, N), np.arange(0, 70)]))
    idx = torch.from_numpy(rows).cuda()
    ref, ab = oracle.gemm_bias_act(A[idx].cpu().numpy(), W, b, True, want_abs=True)
    assert_parity(out[idx].cpu().numpy(), ref, ab, "2^31+ elements GEMM, sampled rows")
    assert not torch.isnan(out).any()
