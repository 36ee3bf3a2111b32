"""CPU-side checks of the C-ABI library: symbols, argument validation, and the host functions
(renumbering, AES rule, GCN weights, CSR relabelling) against the oracle, byte for byte."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2006_06608_amd as gnn
from gnn_synth import config_graph
from util import csr_from_edges, random_sym_csr, read_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["gnn.h", "gnn_bench.h"]
    declared = set()
    for h in headers:
        declared |= set(re.findall(r"\b(gnn_[a-z0-9_]+)\s*\(", open(h).read()))
    assert declared, "no declarations found"
    lib = gnn.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(gnn.exported_symbols())
    assert gnn.gnn_version() >= 100
    assert gnn.gnn_strerror(0) == "ok" and "CSR" in gnn.gnn_strerror(-2)


def test_header_is_plain_c():
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    for h in ("gnn.h", "gnn_bench.h"):
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                            os.path.join(ROOT, "include", h)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_host_argument_validation():
    lib = gnn.load()
    rp = np.array([0, 1, 2], dtype=np.int32)
    ci = np.array([1, 0], dtype=np.int32)
    perm = np.zeros(2, dtype=np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.gnn_reorder(ctypes.c_int32(2), p(rp), p(ci), None, p(perm), None, None, 0) == -1
    assert lib.gnn_reorder(ctypes.c_int32(-1), p(rp), p(ci), p(perm), p(perm), None, None, 0) == -1
    bad = np.array([0, 2, 1], dtype=np.int32)
    assert lib.gnn_reorder(ctypes.c_int32(2), p(bad), p(ci), p(perm), p(perm), None, None, 0) == -2
    oob = np.array([1, 5], dtype=np.int32)
    assert lib.gnn_reorder(ctypes.c_int32(2), p(rp), p(oob), p(perm), p(perm), None, None, 0) == -2
    notzero = np.array([1, 1, 2], dtype=np.int32)
    assert lib.gnn_gcn_norm(ctypes.c_int32(2), p(notzero), p(ci), p(np.zeros(2, np.float32))) == -2
    # device entry points reject bad scalars before touching the GPU
    assert lib.gnn_aggregate_gcn(ctypes.c_int32(4), ctypes.c_int64(4), None, None, None, None, None,
                                 ctypes.c_int32(16), 0, 0, 0, 0, None, ctypes.c_size_t(0), None) == -1
    assert lib.gnn_partition_build(ctypes.c_int32(4), ctypes.c_int64(4), None, ctypes.c_int32(0), None,
                                   ctypes.c_size_t(0), None) == -1
    assert lib.gnn_update_gemm(ctypes.c_int32(4), ctypes.c_int32(0), ctypes.c_int32(4), None, None, None, 0, None,
                               None) == -1
    assert gnn.gnn_workspace_bytes(1000, 5000, 0, 4) >= 256 + 4 * 1001 + 16 * (5000 // 4)
    assert gnn.gnn_workspace_bytes(1000, 5000, 64, 4) >= gnn.gnn_workspace_bytes(1000, 5000, 0, 4) + 1000 * 64 * 4


def test_reorder_hand_trace_and_rule():
    g = read_golden("reorder_trace.txt")
    edges = [tuple(int(x) for x in t.split("-")) for t in g["edges"][0]]
    rp, ci = csr_from_edges(int(g["n"][0][0]), edges)
    perm, iperm, aes, did = gnn.gnn_reorder(rp, ci)
    assert did and perm.tolist() == [int(x) for x in g["perm"][0]]
    assert iperm.tolist() == [int(x) for x in g["iperm"][0]]
    assert aes == oracle.aes(rp, ci)
    # rule says no -> identity, unless forced
    n = 40000
    rp2, ci2 = csr_from_edges(n, [(i, i + 1) for i in range(n - 1)])
    perm2, iperm2, aes2, did2 = gnn.gnn_reorder(rp2, ci2)
    assert not did2 and aes2 == 1.0 and np.array_equal(perm2, np.arange(n)) and np.array_equal(iperm2, np.arange(n))
    perm3, _, _, did3 = gnn.gnn_reorder(rp2, ci2, force=True)
    assert did3 and np.array_equal(perm3, oracle.reorder(rp2, ci2)[0])


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 1), (3, 1), (4, 1), (5, 1), (4, 16), (5, 16)])
def test_reorder_matches_oracle_bitwise(cfg, shrink):
    """All five configurations at full size (the oracle takes about 3 s on the largest), and two reduced ones."""
    g = config_graph(cfg, shrink=shrink)
    perm, iperm, aes, did = gnn.gnn_reorder(g.rowptr, g.colidx, force=True)
    operm, oiperm = oracle.reorder(g.rowptr, g.colidx)
    assert perm.tobytes() == operm.tobytes()
    assert iperm.tobytes() == oiperm.tobytes()
    assert np.array_equal(np.sort(perm), np.arange(g.n, dtype=np.int32)) and np.array_equal(iperm[perm], np.arange(g.n))
    if shrink == 1:
        rp2, ci2 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm)
        orp, oci = oracle.apply_perm_csr(g.rowptr, g.colidx, operm)
        assert rp2.tobytes() == orp.tobytes() and ci2.tobytes() == oci.tobytes()
    s, a = gnn.gnn_aes(g.rowptr, g.colidx)
    assert s == oracle.aes_sum(g.rowptr, g.colidx) and a == aes
    _, _, _, did_rule = gnn.gnn_reorder(g.rowptr, g.colidx)
    assert did_rule == oracle.should_reorder(g.rowptr, g.colidx)


def test_reorder_handles_unsorted_rows_duplicates_and_loops():
    rng = np.random.default_rng(5)
    rp, ci = random_sym_csr(80, 0.08, rng, self_loops=True)
    # shuffle inside rows and duplicate some entries
    rows = [list(ci[rp[i]:rp[i + 1]]) for i in range(80)]
    for r in rows:
        rng.shuffle(r)
        if r:
            r.append(r[0])
    rp2 = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    ci2 = np.asarray([c for r in rows for c in r], dtype=np.int32)
    a = gnn.gnn_reorder(rp, ci, force=True)[0]
    b = gnn.gnn_reorder(rp2, ci2, force=True)[0]
    assert np.array_equal(a, b) and np.array_equal(a, oracle.reorder(rp2, ci2)[0])


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 1), (4, 16)])
def test_gcn_norm_and_relabel_match_oracle_bitwise(cfg, shrink):
    g = config_graph(cfg, shrink=shrink)
    ew = gnn.gnn_gcn_norm(g.rowptr, g.colidx)
    assert ew.tobytes() == oracle.gcn_norm(g.rowptr, g.colidx).tobytes()
    perm = gnn.gnn_reorder(g.rowptr, g.colidx, force=True)[0]
    rp2, ci2, v2 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm, ew)
    orp, oci, ov = oracle.apply_perm_csr(g.rowptr, g.colidx, perm, ew)
    assert rp2.tobytes() == orp.tobytes() and ci2.tobytes() == oci.tobytes() and v2.tobytes() == ov.tobytes()
    rp3, ci3 = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm)
    assert rp3.tobytes() == orp.tobytes() and ci3.tobytes() == oci.tobytes()
    with pytest.raises(gnn.GnnError):
        gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, np.zeros(g.n, dtype=np.int32))  # not a bijection


def test_paper_model_literal_and_decide_ranges():
    assert gnn.gnn_paper_model(16, 32, 128, 3) == (oracle.eq6_dw(16, 32), oracle.eq5_wpt(3, 16, 16), oracle.eq5_smem(128, 32, 16))
    assert gnn.gnn_paper_model(64, 32, 128, 32) == (32, 64.0, 1024)
    for n, nnz, dim in [(2708, 13264, 16), (19717, 108365, 3), (44246, 165028, 64), (410236, 5289110, 96),
                        (1 << 20, 16085932, 64), (1000, 5000, 22), (1000, 5000, 1323)]:
        ngs, dw, wpb = gnn.gnn_decide(n, nnz, 0, dim)
        assert 1 <= ngs <= 128 and 1 <= wpb <= 16
        assert 1 <= dw <= 64 and dw & (dw - 1) == 0


def test_the_models_own_choice_always_fits_the_scratch_memory_of_a_block():
    """Eq. 5's second constraint re-derived: whatever the graph and the row width (up to 15,000 floats),
    the automatic (ngs, dw, waves per block) need at most 64 KB of scratch memory per block (formula of
    gnn.h), also when the caller fixes one or two of the three."""
    rng = np.random.default_rng(0)

    def need(dim, ngs, dw, wpb):
        T = wpb * (64 // dw)
        return -(-4 * 2 * (T * ngs + 8) // 16) * 16 + 4 * wpb * dim + 128 + 256 * wpb

    dims = list(range(1, 70)) + [96, 100, 128, 200, 256, 500, 512, 1000, 1024, 1433, 2048, 3703, 4096, 8192, 12000, 15000]
    for dim in dims:
        for _ in range(6):
            n = int(rng.integers(1, 2_000_000))
            nnz = int(n * rng.choice([0.0, 0.5, 3.7, 15.0, 60.0, 500.0]))
            ngs, dw, wpb = gnn.gnn_decide(n, nnz, int(rng.choice([0, 3, 40, 100000])), dim)
            assert 1 <= ngs <= 128 and 1 <= wpb <= 16 and dw in (1, 2, 4, 8, 16, 32, 64)
            assert need(dim, ngs, dw, wpb) <= 65536, (dim, n, nnz, ngs, dw, wpb)
            # the caller fixes the group size (a sweep): the rest still fits
            ngs2 = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
            g2, dw2, wpb2 = gnn.gnn_decide(n, nnz, 0, dim, ngs=ngs2)
            assert g2 == ngs2 and need(dim, g2, dw2, wpb2) <= 65536, (dim, n, nnz, g2, dw2, wpb2)
    # a caller's own values are kept, bad ones refused
    assert gnn.gnn_decide(1000, 5000, 0, 64, 8, 4, 2) == (8, 4, 2)
    with pytest.raises(gnn.GnnError):
        gnn.gnn_decide(1000, 5000, 0, 64, dw=3)
    with pytest.raises(gnn.GnnError):
        gnn.gnn_decide(1000, 5000, 0, 64, waves_per_block=17)
