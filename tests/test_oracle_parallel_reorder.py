"""Pins for the oracle of the round-based renumbering (oracle/parallel_reorder.py; the loop form is the
oracle, the numpy form its cross-check for large graphs): hand-worked
examples, properties every renumbering must have, recovery of planted communities, and the
locality it buys compared with the sequential merge order."""
import numpy as np
import pytest

import oracle
from gnn_synth import config_graph
from util import csr_from_edges


def _csr(n, undirected):
    return csr_from_edges(n, [(int(a), int(b)) for a, b in undirected])


def test_path_of_three_nodes_worked_by_hand():
    # 0 - 1 - 2: M2 = 4, degrees 1, 2, 1, every score 1*4 - 1*2 = 2.  First pass: 0 -> 1, 1 -> 0 (smallest id among
    # equals), 2 -> 1; 0 and 1 propose to each other, 0 stays and 1 joins it; 2 waits because 1 moves.
    # Second pass: {0,1} (degree 3) and {2}: 1*4 - 3*1 = 1 > 0, they propose to each other, 2 joins.  Order 0, 1, 2.
    rp, ci = _csr(3, [(0, 1), (1, 2)])
    perm, iperm, rounds = oracle.parallel_reorder(rp, ci)
    assert perm.tolist() == [0, 1, 2] and iperm.tolist() == [0, 1, 2] and rounds == 2


def test_path_with_the_middle_node_numbered_last_worked_by_hand():
    # 0 - 2 - 1: 0 -> 2, 1 -> 2, 2 -> 0 (smallest id among equals).  0 and 2 propose to each other: 0 stays,
    # 2 joins 0 and gets position 1; node 1 waits (its target moves).  Second pass: {0,2} and {1}: 4 - 3 > 0, 1 joins
    # at position 2.  New ids: node 0 -> 0, node 2 -> 1, node 1 -> 2.
    rp, ci = _csr(3, [(0, 2), (2, 1)])
    perm, iperm, rounds = oracle.parallel_reorder(rp, ci)
    assert perm.tolist() == [0, 2, 1] and iperm.tolist() == [0, 2, 1] and rounds == 2


def test_two_triangles_joined_by_one_edge_stay_two_communities():
    # triangles {0,2,4} and {1,3,5}, bridge 4 - 1: M2 = 14.  Once each triangle is one community (total degree 7
    # each, one edge between them) the score is 1*14 - 7*7 < 0: no further merge.  New ids keep each triangle
    # together, the one with the smaller root first.
    rp, ci = _csr(6, [(0, 2), (2, 4), (0, 4), (1, 3), (3, 5), (1, 5), (4, 1)])
    perm, _, _ = oracle.parallel_reorder(rp, ci)
    assert sorted(perm[[0, 2, 4]].tolist()) == [0, 1, 2]
    assert sorted(perm[[1, 3, 5]].tolist()) == [3, 4, 5]


def test_no_edges_no_change_and_self_loops_and_duplicates_are_ignored():
    rp = np.zeros(6, dtype=np.int32)
    perm, iperm, rounds = oracle.parallel_reorder(rp, np.zeros(0, dtype=np.int32))
    assert perm.tolist() == list(range(5)) and rounds == 0
    # the path 0 - 2 - 1 again, with self loops and every entry stored twice
    rows = [[0, 0, 2, 2], [1, 2, 2, 1], [0, 1, 2, 0, 1]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.concatenate(rows).astype(np.int32)
    assert oracle.parallel_reorder(rp, ci)[0].tolist() == [0, 2, 1]


@pytest.mark.parametrize("form", ["loop", "numpy"])
def test_hand_worked_examples_hold_for_both_forms(form):
    f = oracle.parallel_reorder if form == "loop" else oracle.parallel_reorder_numpy
    assert f(*_csr(3, [(0, 1), (1, 2)]))[0].tolist() == [0, 1, 2]
    perm, iperm, rounds = f(*_csr(3, [(0, 2), (2, 1)]))
    assert perm.tolist() == [0, 2, 1] and iperm.tolist() == [0, 2, 1] and rounds == 2
    perm, _, _ = f(*_csr(6, [(0, 2), (2, 4), (0, 4), (1, 3), (3, 5), (1, 5), (4, 1)]))
    assert sorted(perm[[0, 2, 4]].tolist()) == [0, 1, 2] and sorted(perm[[1, 3, 5]].tolist()) == [3, 4, 5]


@pytest.mark.parametrize("seed", range(12))
def test_numpy_form_equals_the_loop_form_on_small_random_graphs(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 40))
    m = int(rng.integers(1, 4 * n))
    a, b = rng.integers(0, n, size=m), rng.integers(0, n, size=m)
    rp, ci = _csr(n, zip(a, b))
    perm, iperm, rounds = oracle.parallel_reorder(rp, ci)
    assert np.array_equal(np.sort(perm), np.arange(n)) and np.array_equal(iperm[perm], np.arange(n))
    fast = oracle.parallel_reorder_numpy(rp, ci)
    assert np.array_equal(perm, fast[0]) and np.array_equal(iperm, fast[1]) and rounds == fast[2]
    assert np.array_equal(perm, oracle.parallel_reorder(rp, ci)[0])  # deterministic


@pytest.mark.parametrize("name,cfg,shrink", [("citation", 1, 1), ("batch", 3, 8), ("community", 4, 64), ("rmat", 5, 128)])
def test_numpy_form_equals_the_loop_form_on_graphs_of_thousands_of_nodes(name, cfg, shrink):
    g = config_graph(cfg, shrink=shrink)
    assert g.n >= 2000
    perm, iperm, rounds = oracle.parallel_reorder(g.rowptr, g.colidx)
    fast = oracle.parallel_reorder_numpy(g.rowptr, g.colidx)
    assert np.array_equal(perm, fast[0]) and np.array_equal(iperm, fast[1]) and rounds == fast[2]
    assert rounds >= 3


def test_max_rounds_cuts_both_forms_at_the_same_state():
    g = config_graph(1)
    for r in (1, 2, 5):
        a = oracle.parallel_reorder(g.rowptr, g.colidx, max_rounds=r)
        b = oracle.parallel_reorder_numpy(g.rowptr, g.colidx, max_rounds=r)
        assert a[2] == r and np.array_equal(a[0], b[0]) and b[2] == r


def test_planted_cliques_come_out_contiguous():
    rng = np.random.default_rng(5)
    k, c = 12, 8
    n = k * c
    label = rng.permutation(n)  # shuffled ids
    e = [(label[q * k + a], label[q * k + b]) for q in range(c) for a in range(k) for b in range(a + 1, k)]
    e += [(label[q * k], label[((q + 1) % c) * k + 1]) for q in range(c)]  # a ring of single edges between cliques
    rp, ci = _csr(n, e)
    perm, _, _ = oracle.parallel_reorder(rp, ci)
    for q in range(c):
        new = perm[label[q * k:(q + 1) * k]]
        assert new.max() - new.min() == k - 1, f"clique {q} scattered: {sorted(new.tolist())}"


def test_locality_gain_matches_the_sequential_merge_order():
    g = config_graph(4, shrink=32)  # planted communities, shuffled ids
    perm, _, rounds = oracle.parallel_reorder(g.rowptr, g.colidx)
    rp2, ci2 = oracle.apply_perm_csr(g.rowptr, g.colidx, perm)
    seq = oracle.reorder(g.rowptr, g.colidx)[0]
    rp3, ci3 = oracle.apply_perm_csr(g.rowptr, g.colidx, seq)
    before, after, after_seq = oracle.aes(g.rowptr, g.colidx), oracle.aes(rp2, ci2), oracle.aes(rp3, ci3)
    assert after < 0.5 * before            # Eq. 4 falls by more than half on a community graph
    assert after < 1.15 * after_seq        # and about as far as with the sequential schedule
    assert 1 <= rounds <= 32


def test_aggregation_is_invariant_under_the_new_numbering():
    g = config_graph(2, shrink=8)
    perm, iperm, _ = oracle.parallel_reorder(g.rowptr, g.colidx)
    X = np.ones((g.n, 4), dtype=np.float32)
    rp2, ci2 = oracle.apply_perm_csr(g.rowptr, g.colidx, perm)
    a = oracle.aggregate_gin(g.rowptr, g.colidx, 0.0, X)
    b = oracle.aggregate_gin(rp2, ci2, 0.0, oracle.permute_rows(X, perm))
    assert np.array_equal(oracle.permute_rows(b, iperm), a)  # sums of small integers: exact
