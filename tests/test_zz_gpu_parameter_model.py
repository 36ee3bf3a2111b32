"""The parameter model (Sec. 6, re-derived for this GPU) against measurement, the way Sec. 7.5 of the
paper validates its own: the configuration the model picks must run close to the best of a sweep
over the neighbor-group size and the dimension workers.  Timing test: the margins are wide, and the
file name makes it the last one collected, so that a noisy machine cannot hide other tests."""
import numpy as np
import pytest
import torch

import paper_2006_06608_amd as gnn
from gnn_synth import BASE_SEED, config_graph, features, replicate

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DeviceGraph, dev

# A timing assertion inside a test suite has to survive a noisy machine: the hard bound is loose, the
# measured distances from the best point of the sweep are printed (and quoted in the design notes).
MARGIN = 1.5


def _time_us(fn, reps=5, rounds=3):
    """Best of `rounds` means over `reps` calls: a disturbance from outside lengthens a run, never shortens it."""
    for _ in range(2):
        fn()
    best = float("inf")
    for _ in range(rounds):
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) / reps * 1e3)
    return best


def _sweep(g, dim, eps, ew, ngs_list, dw_list):
    G = DeviceGraph(g.rowptr, g.colidx, ew)
    X = dev(features(g.n, dim, BASE_SEED))
    out = torch.empty_like(X)
    times = {}
    for ngs in ngs_list:
        ws = gnn.alloc_workspace(G.n, G.nnz, dim, ngs)
        gnn.gnn_partition_build(G.n, G.nnz, G.rowptr, ngs, ws)
        for dw in dw_list:
            if ew is None:
                call = gnn.AggregateCall(G.n, G.nnz, G.rowptr, G.colidx, None, eps, X, out, dim, ngs, dw, 0,
                                         gnn.GNN_FLAG_REUSE_PARTITION, ws)
            else:
                call = gnn.AggregateCall(G.n, G.nnz, G.rowptr, G.colidx, G.ew, None, X, out, dim, ngs, dw, 0,
                                         gnn.GNN_FLAG_REUSE_PARTITION, ws)
            times[(ngs, dw)] = _time_us(call)
            gnn.gnn_workspace_status(ws)
        del ws
    return times


class _Graph:
    pass


def _dense_graph(n, deg, seed):
    """Every row has `deg` entries drawn uniformly (a dense graph: mean row 500)."""
    rng = np.random.default_rng(seed)
    g = _Graph()
    g.n, g.nnz = n, n * deg
    g.rowptr = (np.arange(n + 1, dtype=np.int64) * deg).astype(np.int32)
    g.colidx = np.sort(rng.integers(0, n, size=(n, deg), dtype=np.int32), axis=1).reshape(-1)
    return g


def _renumbered(g):
    perm = gnn.gnn_reorder(g.rowptr, g.colidx, force=True)[0]
    h = _Graph()
    h.n, h.nnz = g.n, g.nnz
    h.rowptr, h.colidx = gnn.gnn_apply_perm_csr(g.rowptr, g.colidx, perm)
    return h


# name -> (graph, Dim, kind); the first three are the workloads the model's constants were first set on, the
# others were not used for that
_CASES = {
    "rmat_gin_dim64": (lambda: config_graph(5), 64, "gin"),
    "community_gcn_dim96": (lambda: config_graph(4), 96, "gcn"),
    "small_graph_batch_gin_dim64": (lambda: replicate(config_graph(3), 8), 64, "gin"),
    "citation_gcn_dim16": (lambda: config_graph(2), 16, "gcn"),
    "citation_gcn_dim3": (lambda: config_graph(2), 3, "gcn"),
    "community_gcn_dim16": (lambda: config_graph(4), 16, "gcn"),
    "community_gcn_dim22": (lambda: config_graph(4), 22, "gcn"),
    "dense_rows_of_500_gin_dim64": (lambda: _dense_graph(20000, 500, 1), 64, "gin"),
    "community_renumbered_gcn_dim128": (lambda: _renumbered(config_graph(4)), 128, "gcn"),
    "community_renumbered_gcn_dim256": (lambda: _renumbered(config_graph(4)), 256, "gcn"),
}


@pytest.mark.parametrize("case", list(_CASES))
def test_model_choice_is_close_to_the_best_of_the_sweep(case):
    make, dim, kind = _CASES[case]
    g = make()
    eps = 0.0 if kind == "gin" else None
    ew = gnn.gnn_gcn_norm(g.rowptr, g.colidx) if kind == "gcn" else None
    ngs_m, dw_m, _ = gnn.gnn_decide(g.n, g.nnz, 0, dim)
    ngs_list = sorted({4, 16, 32, 64, ngs_m} | ({2, 8} if case == "rmat_gin_dim64" else set()))
    vec = 4 if dim % 4 == 0 else (2 if dim % 2 == 0 else 1)
    units = -(-dim // vec)
    dw_list = [0] + [d for d in (2, 4, 8, 16, 32, 64) if d <= 2 * units and -(-units // d) <= 4]
    times = _sweep(g, dim, eps, ew, ngs_list, dw_list)
    picked = times[(ngs_m, 0)]
    best_key = min(times, key=times.get)
    best = times[best_key]
    print(f"{case}: model (ngs {ngs_m}, dw {dw_m}) {picked:.1f} us; best {best_key} {best:.1f} us "
          f"({100 * (picked / best - 1):.1f} % off); " + ", ".join(f"{k}: {v:.0f}" for k, v in sorted(times.items())), flush=True)
    assert picked <= MARGIN * best, f"{case}: model's pick {picked:.1f} us against {best:.1f} us at {best_key}"
    # the paper's observation (Sec. 7.5): very small groups are far from the optimum (where the kernel
    # is not bound by its launch)
    if best > 30.0:
        assert times[(min(ngs_list), 0)] > picked
