"""Seeded random graphs shaped like the three graph types of Table 1 of the paper.

Every graph is returned as a CSR pair (rowptr int32[n+1], colidx int32[nnz]) with
sorted, duplicate-free rows.  All graphs are symmetric (an undirected edge is two
stored entries).  Nothing here computes anything the method computes: edge weights,
aggregation and renumbering live elsewhere.

The five numbered configurations stand in for public datasets that are not
available offline (small citation graphs, a batch of small molecule-like graphs, a
large co-purchase graph, and an R-MAT graph); only their sizes and degree
distributions are taken.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 20060660800


@dataclass
class Graph:
    n: int
    rowptr: np.ndarray  # int32 [n+1]
    colidx: np.ndarray  # int32 [nnz]
    name: str = ""
    meta: Dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr).astype(np.int64)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(stream)])))


# ----------------------------------------------------------------------------- CSR builders
def _csr_from_directed(n: int, src: np.ndarray, dst: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Sort directed entries by (src, dst); the caller guarantees there are no duplicates."""
    key = src.astype(np.int64) * np.int64(n) + dst.astype(np.int64)
    key.sort()
    s = (key // n).astype(np.int64)
    colidx = (key % n).astype(np.int32)
    counts = np.bincount(s, minlength=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    return rowptr.astype(np.int32), colidx


def _unique_undirected(n: int, u: np.ndarray, v: np.ndarray, limit: Optional[int] = None):
    """Distinct undirected pairs (loops dropped) in order of first appearance."""
    keep = u != v
    u, v = u[keep], v[keep]
    lo = np.minimum(u, v).astype(np.int64)
    hi = np.maximum(u, v).astype(np.int64)
    key = lo * np.int64(n) + hi
    _, first = np.unique(key, return_index=True)
    first.sort()
    if limit is not None:
        first = first[:limit]
    return lo[first], hi[first]


def csr_from_undirected_pairs(n: int, lo: np.ndarray, hi: np.ndarray, self_loops: bool = False):
    """Symmetric CSR from distinct undirected pairs; optionally one self loop per node."""
    src = np.concatenate([lo, hi])
    dst = np.concatenate([hi, lo])
    if self_loops:
        ids = np.arange(n, dtype=np.int64)
        src = np.concatenate([src, ids])
        dst = np.concatenate([dst, ids])
    return _csr_from_directed(n, src, dst)


def _upper_pairs(g: Graph):
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    cols = g.colidx.astype(np.int64)
    keep = rows < cols
    return rows[keep], cols[keep]


def add_self_loops(g: Graph) -> Graph:
    """The graph with one (i, i) entry added to every row that has none."""
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    cols = g.colidx.astype(np.int64)
    keep = rows != cols
    ids = np.arange(g.n, dtype=np.int64)
    rp, ci = _csr_from_directed(g.n, np.concatenate([rows[keep], ids]), np.concatenate([cols[keep], ids]))
    return Graph(g.n, rp, ci, g.name + "+I", dict(g.meta, self_loops=True))


def shuffle_ids(g: Graph, seed: int, stream: int = 99) -> Tuple[Graph, np.ndarray]:
    """Relabel nodes by a seeded random bijection; returns (graph, label) with label[old] = new."""
    label = _rng(seed, stream).permutation(g.n).astype(np.int64)
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    rp, ci = _csr_from_directed(g.n, label[rows], label[g.colidx.astype(np.int64)])
    return Graph(g.n, rp, ci, g.name + "/shuffled", dict(g.meta, shuffled=True)), label.astype(np.int32)


# ----------------------------------------------------------------------------- degree weights
def _power_law_weights(n: int, two_m: int, exponent: float, max_degree: float) -> np.ndarray:
    """theta_i ~ (i + i0)^(-1/(exponent-1)), scaled to sum to two_m, i0 set so theta_0 ~ max_degree."""
    alpha = 1.0 / (exponent - 1.0)
    idx = np.arange(n, dtype=np.float64)

    def top(i0):
        w = (idx + i0) ** (-alpha)
        return two_m * w[0] / w.sum()

    lo, hi = 1e-3, float(n)
    if top(lo) <= max_degree:
        i0 = lo
    else:
        for _ in range(80):
            mid = np.sqrt(lo * hi)
            if top(mid) > max_degree:
                lo = mid
            else:
                hi = mid
        i0 = hi
    w = (idx + i0) ** (-alpha)
    return w * (two_m / w.sum())


def _sample_until(n: int, m_target: int, draw):
    """Call draw(k) -> (u, v) until m_target distinct undirected pairs exist; keep the first m_target."""
    lo_all = np.empty(0, dtype=np.int64)
    hi_all = np.empty(0, dtype=np.int64)
    for _ in range(64):
        need = m_target - lo_all.size
        if need <= 0:
            break
        k = int(need * 1.25) + 1024
        u, v = draw(k)
        lo, hi = _unique_undirected(n, np.concatenate([lo_all, np.minimum(u, v)]),
                                    np.concatenate([hi_all, np.maximum(u, v)]), limit=m_target)
        lo_all, hi_all = lo, hi
    assert lo_all.size == m_target, "could not reach the requested number of edges"
    return lo_all, hi_all


def power_law_graph(n: int, m_undirected: int, exponent: float, max_degree: float,
                    seed: int, name: str = "powerlaw") -> Graph:
    """Chung-Lu style symmetric graph with exactly m_undirected edges and random node ids."""
    rng = _rng(seed, 1)
    theta = _power_law_weights(n, 2 * m_undirected, exponent, max_degree)
    label = rng.permutation(n).astype(np.int64)  # hubs get random ids
    cdf = np.cumsum(theta)
    cdf /= cdf[-1]

    def draw(k):
        u = np.minimum(np.searchsorted(cdf, rng.random(k), side="right"), n - 1)
        v = np.minimum(np.searchsorted(cdf, rng.random(k), side="right"), n - 1)
        return label[u], label[v]

    lo, hi = _sample_until(n, m_undirected, draw)
    rp, ci = csr_from_undirected_pairs(n, lo, hi)
    return Graph(n, rp, ci, name, {"exponent": exponent, "m_undirected": m_undirected})


def planted_community_graph(n: int, m_undirected: int, exponent: float, max_degree: float,
                            p_in: float, comm_min: int, comm_max: int, seed: int,
                            name: str = "planted") -> Graph:
    """Degree-corrected block model: power-law degrees, power-law community sizes.

    Node ids come out community-contiguous (the 'already block-diagonal' labelling);
    use shuffle_ids for the irregular labelling.
    """
    rng = _rng(seed, 2)
    # community sizes ~ s^-2 on [comm_min, comm_max]
    sizes = []
    total = 0
    while total < n:
        r = rng.random()
        s = int(1.0 / (1.0 / comm_min - r * (1.0 / comm_min - 1.0 / comm_max)))
        s = max(comm_min, min(comm_max, s))
        s = min(s, n - total)
        sizes.append(s)
        total += s
    sizes = np.asarray(sizes, dtype=np.int64)
    ends = np.cumsum(sizes)
    starts = ends - sizes
    comm = np.repeat(np.arange(sizes.size, dtype=np.int64), sizes)

    theta = _power_law_weights(n, 2 * m_undirected, exponent, max_degree)
    theta = theta[rng.permutation(n)]  # hubs spread over communities
    cdf = np.cumsum(theta)
    tot = cdf[-1]
    cdf0 = np.concatenate([[0.0], cdf])

    def draw(k):
        u = np.minimum(np.searchsorted(cdf, rng.random(k) * tot, side="right"), n - 1)
        inside = rng.random(k) < p_in
        c = comm[u]
        lo_w = np.where(inside, cdf0[starts[c]], 0.0)
        hi_w = np.where(inside, cdf0[ends[c]], tot)
        r = lo_w + rng.random(k) * (hi_w - lo_w)
        v = np.searchsorted(cdf, r, side="right")
        v = np.where(inside, np.clip(v, starts[c], ends[c] - 1), np.minimum(v, n - 1))
        return u.astype(np.int64), v.astype(np.int64)

    lo, hi = _sample_until(n, m_undirected, draw)
    rp, ci = csr_from_undirected_pairs(n, lo, hi)
    return Graph(n, rp, ci, name, {"communities": int(sizes.size), "p_in": p_in, "exponent": exponent})


def block_diagonal_batch(num_graphs: int, mean_nodes: float, edge_factor: float, max_deg: int,
                         seed: int, name: str = "batch") -> Graph:
    """Disjoint small graphs with consecutive ids per graph: spanning tree + random extra edges."""
    rng = _rng(seed, 3)
    sigma = 0.6
    mu = np.log(mean_nodes) - 0.5 * sigma * sigma
    sizes = np.clip(np.rint(rng.lognormal(mu, sigma, num_graphs)), 4, 200).astype(np.int64)
    us, vs = [], []
    base = 0
    for s in sizes:
        s = int(s)
        deg = np.zeros(s, dtype=np.int64)
        have = set()
        for i in range(1, s):  # random tree with a degree cap
            while True:
                j = int(rng.integers(0, i))
                if deg[j] < max_deg:
                    break
            have.add((j, i))
            deg[i] += 1
            deg[j] += 1
        target = min(int(round(edge_factor * s)), s * (s - 1) // 2, (s * max_deg) // 2)
        tries = 0
        while len(have) < target and tries < 50 * target:
            tries += 1
            a = int(rng.integers(0, s))
            b = int(rng.integers(0, s))
            if a == b:
                continue
            a, b = min(a, b), max(a, b)
            if (a, b) in have or deg[a] >= max_deg or deg[b] >= max_deg:
                continue
            have.add((a, b))
            deg[a] += 1
            deg[b] += 1
        e = np.asarray(sorted(have), dtype=np.int64)
        us.append(e[:, 0] + base)
        vs.append(e[:, 1] + base)
        base += s
    n = int(base)
    lo = np.concatenate(us)
    hi = np.concatenate(vs)
    rp, ci = csr_from_undirected_pairs(n, lo, hi)
    return Graph(n, rp, ci, name, {"num_graphs": num_graphs, "graph_sizes": sizes})


def replicate(g: Graph, copies: int) -> Graph:
    """Block-diagonal union of `copies` disjoint copies of g, ids offset per copy (a larger batch of
    the same family: the shape of the paper's big Type II sets, millions of nodes in small graphs)."""
    if copies <= 1:
        return g
    n, nnz = g.n, g.nnz
    assert copies * n < 2 ** 31 and copies * nnz < 2 ** 31
    off_n = (np.arange(copies, dtype=np.int64) * n)[:, None]
    off_e = (np.arange(copies, dtype=np.int64) * nnz)[:, None]
    rp = np.concatenate([(g.rowptr[None, :-1].astype(np.int64) + off_e).ravel(), [copies * nnz]]).astype(np.int32)
    ci = (g.colidx[None, :].astype(np.int64) + off_n).ravel().astype(np.int32)
    return Graph(copies * n, rp, ci, f"{g.name}x{copies}", {"copies": copies})


def rmat_graph(scale: int, n_pairs: int, a: float, b: float, c: float, seed: int,
               scramble: bool = True, name: str = "rmat") -> Graph:
    """R-MAT: n_pairs sampled undirected pairs on 2^scale nodes, symmetrised, de-duplicated, loops dropped."""
    rng = _rng(seed, 4)
    n = 1 << scale
    u = np.zeros(n_pairs, dtype=np.int64)
    v = np.zeros(n_pairs, dtype=np.int64)
    for _ in range(scale):
        r = rng.random(n_pairs)
        ubit = r >= a + b
        vbit = ((r >= a) & (r < a + b)) | (r >= a + b + c)
        u = (u << 1) | ubit
        v = (v << 1) | vbit
    if scramble:
        label = rng.permutation(n).astype(np.int64)
        u, v = label[u], label[v]
    lo, hi = _unique_undirected(n, u, v)
    rp, ci = csr_from_undirected_pairs(n, lo, hi)
    return Graph(n, rp, ci, name, {"scale": scale, "pairs": n_pairs, "a": a, "b": b, "c": c,
                                   "scrambled": scramble})


# ----------------------------------------------------------------------------- dense inputs
def features(n: int, dim: int, seed: int, stream: int = 10) -> np.ndarray:
    """X ~ N(0, 1), fp32, row-major [n, dim]."""
    return _rng(seed, stream).standard_normal((n, dim), dtype=np.float32)


def glorot(fan_in: int, fan_out: int, seed: int, stream: int = 20) -> np.ndarray:
    """Glorot-uniform W[fan_in, fan_out], fp32."""
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return _rng(seed, stream).uniform(-lim, lim, size=(fan_in, fan_out)).astype(np.float32)


# ----------------------------------------------------------------------------- the five configurations
_SPECS = {
    1: dict(kind="gcn_agg", n=2708, m=5278, exponent=2.8, max_degree=170, self_loops=True,
            dims=[16], desc="citation-like power-law graph, single GCN aggregation, Dim 16"),
    2: dict(kind="gcn", n=19717, m=44324, exponent=2.6, max_degree=170, self_loops=True,
            dims=[500, 16, 3], desc="citation-like power-law graph, 2-layer GCN 500-16-3"),
    3: dict(kind="gin", num_graphs=1113, mean_nodes=39.06, edge_factor=1.865, max_deg=10,
            self_loops=False, dims=[64] * 6, desc="batch of 1,113 small graphs, 5-layer GIN, Dim 64"),
    4: dict(kind="gcn", n=410236, m=2439437, exponent=2.1, max_degree=30000, p_in=0.85,
            comm_min=100, comm_max=10000, self_loops=True, dims=[96, 16, 22],
            desc="large scale-free graph with planted communities, GCN aggregation Dim 96 and 2-layer GCN 96-16-22"),
    5: dict(kind="gin", scale=20, pairs=8388608, a=0.57, b=0.19, c=0.19, self_loops=False,
            dims=[64] * 6, desc="R-MAT scale 20, 5-layer GIN, Dim 64"),
}


def config_spec(cfg: int) -> Dict:
    return dict(_SPECS[cfg])


def _cache_dir() -> Optional[str]:
    d = os.environ.get("GNN_SYNTH_CACHE", "/tmp/gnn_synth_cache")
    if d in ("", "0", "off"):
        return None
    try:
        os.makedirs(d, exist_ok=True)
    except OSError:
        return None
    return d


def config_graph(cfg: int, shrink: int = 1, variant: str = "default") -> Graph:
    """Graph of configuration cfg (1..5).

    shrink > 1 divides node and edge counts (a smaller graph of the same family, for CPU-sized
    parity cases).  variant: for cfg 4, 'shuffled' (default, irregular ids) or 'planted'
    (community-contiguous ids); for cfg 5, 'scrambled' (default) or 'natural'.
    Self loops are included where the configuration asks for them (the GCN ones).
    """
    spec = _SPECS[cfg]
    seed = BASE_SEED + cfg
    cdir = _cache_dir()
    path = None
    if cdir is not None:
        path = os.path.join(cdir, f"cfg{cfg}_s{shrink}_{variant}.npz")
        if os.path.exists(path):
            try:
                z = np.load(path)
                return Graph(int(z["n"]), z["rowptr"], z["colidx"], str(z["name"]), {"cached": True})
            except Exception:
                pass
    if cfg in (1, 2):
        g = power_law_graph(spec["n"] // shrink, spec["m"] // shrink, spec["exponent"],
                            max(8, spec["max_degree"] // max(1, int(np.sqrt(shrink)))), seed, f"cfg{cfg}")
    elif cfg == 3:
        g = block_diagonal_batch(max(2, spec["num_graphs"] // shrink), spec["mean_nodes"],
                                 spec["edge_factor"], spec["max_deg"], seed, "cfg3")
    elif cfg == 4:
        g = planted_community_graph(spec["n"] // shrink, spec["m"] // shrink, spec["exponent"],
                                    max(16, spec["max_degree"] // max(1, int(np.sqrt(shrink)))), spec["p_in"],
                                    spec["comm_min"], max(spec["comm_min"] + 1, spec["comm_max"] // shrink),
                                    seed, "cfg4")
        if variant in ("default", "shuffled"):
            g, _ = shuffle_ids(g, seed)
    elif cfg == 5:
        sh = int(np.log2(shrink)) if shrink > 1 else 0
        g = rmat_graph(spec["scale"] - sh, spec["pairs"] >> sh, spec["a"], spec["b"], spec["c"], seed,
                       scramble=(variant != "natural"), name="cfg5")
    else:
        raise ValueError(cfg)
    if spec["self_loops"]:
        g = add_self_loops(g)
    if path is not None:
        try:
            tmp = path + f".{os.getpid()}.tmp.npz"
            np.savez(tmp, n=g.n, rowptr=g.rowptr, colidx=g.colidx, name=g.name)
            os.replace(tmp, path)
        except OSError:
            pass
    return g
