"""CPU oracle for the round-based (data-parallel) form of the community renumbering -- TEST
INFRASTRUCTURE ONLY.

Sec. 5.1 of the paper asks for node ids that follow communities found by merging for modularity; it
does not fix the merge schedule.  The GPU library also offers a schedule made of synchronous rounds
(every community looks at the same state), which this file restates in plain Python, integers only,
so that the two can be compared bit for bit.

Two forms of the same schedule live here.  `parallel_reorder` is THE oracle: dictionaries and loops,
one community at a time, each step of the list below written out so that it can be checked by eye;
it serves graphs of up to some ten thousand nodes.  `parallel_reorder_numpy` takes the same steps
with sorts and segmented sums; it is pinned to the loop form (equal permutations on random graphs of
up to a few thousand nodes, tests/test_oracle_parallel_reorder.py) and only stands in for it where
the loop form would take minutes (the full-size community graph).

state    every node belongs to a community, named after one of its nodes (the root); a community
         has a total degree `degw`, a `size`, and an order of its nodes (`pos`, 0-based, root first);
         between communities there are weighted edges (number of original entries, both directions).
per merge round:
      1. score of community u towards a neighbouring community v:
            S(u, v) = w(u, v) * M2 - degw(u) * degw(v)      (M2 = entries of the clean graph; this is
         the modularity gain of the merge up to a positive factor).  u proposes to the v with the
         largest S, the smallest id among equals, provided that S > 0.
      2. two communities that propose to each other: the one with the smaller id stays, the other
         keeps its proposal.
      3. a proposal u -> t is carried out in this round only if t itself does not move (stars only;
         the others try again in the next round, against the new state).
      4. the joiners of t are appended to t's node order by ascending id; sizes and degrees add up;
         the edges are renamed, self edges dropped, parallel edges summed.
end      when a round carries out nothing (or after max_rounds).  New ids: communities by ascending
         root id, inside a community by `pos`.
The clean graph ignores self loops and counts duplicate entries once, as the sequential form does.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

def parallel_reorder(rowptr, colidx, max_rounds: int = 64) -> Tuple[np.ndarray, np.ndarray, int]:
    """Returns perm (old -> new), iperm (new -> old), both int32[n], and the number of rounds that merged."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    n = rowptr.size - 1
    # the clean graph: distinct neighbours other than the node itself, unit weights
    adj = [dict() for _ in range(n)]
    for i in range(n):
        for j in colidx[rowptr[i]:rowptr[i + 1]]:
            if int(j) != i:
                adj[i][int(j)] = 1
    M2 = sum(len(a) for a in adj)
    degw = [len(a) for a in adj]
    members = [[i] for i in range(n)]      # node order of every community, root first
    alive = [True] * n                     # still the root of a community
    rounds = 0
    for _ in range(max_rounds):
        # 1. every community proposes to the neighbour of largest score, the smallest id among equals
        best = list(range(n))
        for u in range(n):
            if not alive[u]:
                continue
            top = None
            for v in sorted(adj[u]):
                s = adj[u][v] * M2 - degw[u] * degw[v]
                if top is None or s > top[0]:
                    top = (s, v)
            if top is not None and top[0] > 0:
                best[u] = top[1]
        # 2. of two communities that propose to each other the smaller id stays
        prop = list(best)
        for u in range(n):
            if best[u] != u and best[best[u]] == u and u < best[u]:
                prop[u] = u
        # 3. only proposals to a community that does not move itself are carried out
        joins = [u for u in range(n) if prop[u] != u and prop[prop[u]] == prop[u]]
        if not joins:
            break
        rounds += 1
        # 4. joiners are appended to their target by ascending id; degrees add up; edges are renamed
        target = {u: prop[u] for u in joins}
        for u in sorted(joins):
            t = target[u]
            members[t] += members[u]
            degw[t] += degw[u]
            alive[u] = False
        new_adj = [dict() for _ in range(n)]
        for u in range(n):
            for v, wt in adj[u].items():
                a, b = target.get(u, u), target.get(v, v)
                if a != b:
                    new_adj[a][b] = new_adj[a].get(b, 0) + wt
        adj = new_adj
    # new ids: communities by ascending root id, inside a community by position
    order = [v for r in range(n) if alive[r] for v in members[r]]
    iperm = np.array(order, dtype=np.int32).reshape(n)
    perm = np.empty(n, dtype=np.int32)
    perm[iperm] = np.arange(n, dtype=np.int32)
    return perm, iperm, rounds


def parallel_reorder_numpy(rowptr, colidx, max_rounds: int = 64) -> Tuple[np.ndarray, np.ndarray, int]:
    """The vectorised cross-check of parallel_reorder (same steps, same result); for large graphs."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    n = rowptr.size - 1
    ids = np.arange(n, dtype=np.int64)
    src = np.repeat(ids, np.diff(rowptr))
    off_diag = src != colidx
    key = np.unique(src[off_diag] * n + colidx[off_diag])
    cu, cv = key // n, key % n
    w = np.ones(key.size, dtype=np.int64)
    M2 = int(key.size)
    degw = np.bincount(cu, minlength=n).astype(np.int64)
    size = np.ones(n, dtype=np.int64)
    pos = np.zeros(n, dtype=np.int64)
    comm = ids.copy()
    rounds = 0
    for _ in range(max_rounds):
        if cu.size == 0:
            break
        # 1. proposals
        S = w * M2 - degw[cu] * degw[cv]
        order = np.lexsort((cv, -S, cu))          # by community, best score first, smallest id first
        head = np.ones(cu.size, dtype=bool)
        head[1:] = cu[order][1:] != cu[order][:-1]
        pu, pv, pS = cu[order][head], cv[order][head], S[order][head]
        best = ids.copy()
        best[pu[pS > 0]] = pv[pS > 0]
        # 2. mutual proposals: the smaller id stays
        stays = (best[best] == ids) & (best != ids) & (ids < best)
        prop = np.where(stays, ids, best)
        # 3. stars only
        joins = (prop != ids) & (prop[prop] == prop)
        if not joins.any():
            break
        rounds += 1
        target = np.where(joins, prop, ids)
        # 4. append the joiners of every target by ascending id
        j = ids[joins]
        t = target[j]
        by_target = np.lexsort((j, t))
        j, t = j[by_target], t[by_target]
        before = np.cumsum(size[j]) - size[j]              # sizes of all joiners sorted before this one
        first = np.ones(j.size, dtype=bool)
        first[1:] = t[1:] != t[:-1]
        group_start = np.maximum.accumulate(np.where(first, before, 0))
        shift = np.zeros(n, dtype=np.int64)
        shift[j] = size[t] + (before - group_start)
        pos += shift[comm]
        comm = target[comm]
        np.add.at(size, t, size[j])
        np.add.at(degw, t, degw[j])
        cu, cv = target[cu], target[cv]
        keep = cu != cv
        key = cu[keep] * n + cv[keep]
        by_key = np.argsort(key, kind="stable")
        key, wk = key[by_key], w[keep][by_key]
        start = np.ones(key.size, dtype=bool)
        start[1:] = key[1:] != key[:-1]
        idx = np.flatnonzero(start)
        w = np.add.reduceat(wk, idx) if idx.size else wk[:0]
        key = key[start]
        cu, cv = key // n, key % n
    roots = ids[comm == ids]
    base = np.zeros(n, dtype=np.int64)
    base[roots] = np.cumsum(size[roots]) - size[roots]
    perm = (base[comm] + pos).astype(np.int32)
    iperm = np.empty(n, dtype=np.int32)
    iperm[perm] = np.arange(n, dtype=np.int32)
    return perm, iperm, rounds
