"""Graph preparation on the device: the round-based renumbering against its oracle, the loop form of oracle/parallel_reorder.py (bit-exact, up to the full-size community graph),
the device CSR relabelling and GCN weights against the oracle (byte-equal), and the whole on-device
pipeline feeding an aggregation."""
import numpy as np
import pytest
import torch

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph, features

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import assert_parity, dev


def _dev_csr(rp, ci):
    rpd = dev(rp.astype(np.int32))
    cid = dev(ci.astype(np.int32)) if ci.size else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
    return rpd, cid


def _graphs():
    yield "cfg1", config_graph(1)
    yield "cfg2", config_graph(2)
    yield "cfg3/8", config_graph(3, shrink=8)
    yield "cfg4/16", config_graph(4, shrink=16)
    yield "cfg5/16", config_graph(5, shrink=16)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3/8", "cfg4/16", "cfg5/16"])
def test_device_renumbering_equals_the_oracle_bit_for_bit(name):
    g = dict(_graphs())[name]
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    perm, iperm, rounds = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid)
    operm, oiperm, orounds = oracle.parallel_reorder(g.rowptr, g.colidx)
    assert rounds == orounds
    assert np.array_equal(perm.cpu().numpy(), operm), f"{name}: permutation differs"
    assert np.array_equal(iperm.cpu().numpy(), oiperm)
    # twice the same
    perm2, _, _ = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid)
    assert torch.equal(perm, perm2)


def test_device_renumbering_full_size_community_graph():
    g = config_graph(4)
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    print(f"device renumbering: n {g.n} nnz {g.nnz}", flush=True)
    perm, iperm, rounds = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid)
    operm, _, orounds = oracle.parallel_reorder(g.rowptr, g.colidx)
    assert rounds == orounds and np.array_equal(perm.cpu().numpy(), operm)
    # the locality it buys (Eq. 4), on the device-relabelled graph
    rp2, ci2 = gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, cid, perm)
    before = gnn.gnn_aes(g.rowptr, g.colidx)[1]
    after = gnn.gnn_aes(rp2.cpu().numpy(), ci2.cpu().numpy())[1]
    assert after < 0.5 * before


def test_self_loops_duplicates_isolated_nodes_and_tiny_graphs():
    # rows unsorted, entries repeated, self loops, nodes without entries
    rows = [[1, 1, 0, 3], [0, 0, 1], [], [0, 3, 3], [], [6], [5, 6, 5]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.concatenate([np.array(r, dtype=np.int32) for r in rows])
    rpd, cid = _dev_csr(rp, ci)
    perm, iperm, rounds = gnn.gnn_reorder_device(len(rows), ci.size, rpd, cid)
    operm, oiperm, orounds = oracle.parallel_reorder(rp, ci)
    assert perm.cpu().numpy().tolist() == operm.tolist() and rounds == orounds
    # no entries at all: identity
    rp0 = np.zeros(6, dtype=np.int32)
    perm, iperm, rounds = gnn.gnn_reorder_device(5, 0, dev(rp0), torch.zeros(1, dtype=torch.int32, device="cuda"))
    assert perm.cpu().numpy().tolist() == [0, 1, 2, 3, 4] and rounds == 0
    # one node with a self loop
    perm, _, _ = gnn.gnn_reorder_device(1, 1, dev(np.array([0, 1], dtype=np.int32)), dev(np.array([0], dtype=np.int32)))
    assert perm.cpu().numpy().tolist() == [0]
    # the round limit is honoured (0 rounds: identity)
    g = config_graph(1)
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    perm, _, rounds = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid, max_rounds=0)
    assert rounds == 0 and np.array_equal(perm.cpu().numpy(), np.arange(g.n))
    perm, _, rounds = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid, max_rounds=2)
    assert rounds == 2 and np.array_equal(perm.cpu().numpy(), oracle.parallel_reorder(g.rowptr, g.colidx, max_rounds=2)[0])


@pytest.mark.parametrize("name", ["cfg1", "cfg4/16", "cfg5/16"])
def test_device_relabel_and_weights_equal_the_oracle_byte_for_byte(name):
    g = dict(_graphs())[name]
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    ew = gnn.gnn_gcn_norm_device(g.n, g.nnz, rpd, cid)
    oew = oracle.gcn_norm(g.rowptr, g.colidx)
    assert ew.cpu().numpy().tobytes() == oew.tobytes()
    perm = oracle.reorder(g.rowptr, g.colidx)[0]
    rp2, ci2, v2 = gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, cid, dev(perm), ew)
    orp, oci, ov = oracle.apply_perm_csr(g.rowptr, g.colidx, perm, oew)
    assert rp2.cpu().numpy().tobytes() == orp.tobytes()
    assert ci2.cpu().numpy().tobytes() == oci.tobytes()
    assert v2.cpu().numpy().tobytes() == ov.tobytes()
    rp3, ci3 = gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, cid, dev(perm))
    assert torch.equal(rp3, rp2) and torch.equal(ci3, ci2)


@pytest.mark.parametrize("name", ["cfg1", "cfg3/8", "cfg4/16", "cfg5/16"])
def test_device_aes_and_rule_equal_the_oracle(name):
    g = dict(_graphs())[name]
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    total, mean, want = gnn.gnn_aes_device(g.n, g.nnz, rpd, cid)
    assert total == oracle.aes_sum(g.rowptr, g.colidx)
    assert mean == oracle.aes(g.rowptr, g.colidx)
    assert want == oracle.should_reorder(g.rowptr, g.colidx)


def test_device_transpose_equals_the_oracle_byte_for_byte():
    # a directed graph (not its own transpose) with values
    rng = np.random.default_rng(3)
    n, m = 5000, 60000
    src, dst = rng.integers(0, n, size=m), rng.integers(0, n, size=m)
    order = np.lexsort((dst, src))
    src, dst = src[order], dst[order]
    rp = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(src, minlength=n), out=rp[1:])
    ci = dst.astype(np.int32)
    val = rng.standard_normal(m).astype(np.float32)
    rpd, cid = _dev_csr(rp, ci)
    rpt, cit, vt = gnn.gnn_csr_transpose_device(n, m, rpd, cid, dev(val))
    orp, oci, ov = oracle.csr_transpose(rp, ci, val)
    assert rpt.cpu().numpy().tobytes() == orp.astype(np.int32).tobytes()
    assert cit.cpu().numpy().tobytes() == oci.astype(np.int32).tobytes()
    assert vt.cpu().numpy().tobytes() == ov.astype(np.float32).tobytes()
    rpt2, cit2 = gnn.gnn_csr_transpose_device(n, m, rpd, cid)
    assert torch.equal(rpt2, rpt) and torch.equal(cit2, cit)


def test_errors_are_reported():
    g = config_graph(1)
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    with pytest.raises(gnn.GnnError):  # not a bijection
        gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, cid, torch.zeros(g.n, dtype=torch.int32, device="cuda"))
    bad = cid.clone()
    bad[5] = g.n  # column index out of range
    with pytest.raises(gnn.GnnError):
        gnn.gnn_reorder_device(g.n, g.nnz, rpd, bad)
    with pytest.raises(gnn.GnnError):
        gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, bad, dev(np.arange(g.n, dtype=np.int32)))


def test_whole_preparation_on_the_device_then_aggregation():
    g = config_graph(4, shrink=16)
    X = features(g.n, 32, seed=8)
    rpd, cid = _dev_csr(g.rowptr, g.colidx)
    gnn.gnn_validate_csr_device(g.n, g.nnz, rpd, cid)
    ew = gnn.gnn_gcn_norm_device(g.n, g.nnz, rpd, cid)
    perm, iperm, _ = gnn.gnn_reorder_device(g.n, g.nnz, rpd, cid)
    rp2, ci2, ew2 = gnn.gnn_apply_perm_csr_device(g.n, g.nnz, rpd, cid, perm, ew)
    Xd = dev(X)
    Xp = torch.empty_like(Xd)
    gnn.gnn_permute_rows(g.n, 32, perm, Xd, Xp)
    outp = torch.full_like(Xd, float("nan"))
    ws = gnn.alloc_workspace(g.n, g.nnz, 32, 0)
    gnn.gnn_aggregate_gcn(g.n, g.nnz, rp2, ci2, ew2, Xp, outp, 32, workspace=ws)
    out = torch.empty_like(outp)
    gnn.gnn_permute_rows(g.n, 32, iperm, outp, out)  # back to the original numbering
    torch.cuda.synchronize()
    gnn.gnn_workspace_status(ws)
    ref, ab = oracle.aggregate_gcn(g.rowptr, g.colidx, oracle.gcn_norm(g.rowptr, g.colidx), X, want_abs=True)
    assert_parity(out.cpu().numpy(), ref, ab, "aggregation after the on-device preparation")
