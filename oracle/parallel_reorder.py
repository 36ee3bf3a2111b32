"""CPU oracle for the round-based (data-parallel) form of the community renumbering -- TEST
INFRASTRUCTURE ONLY.

Sec. 5.1 of the paper asks for node ids that follow communities found by merging for modularity; it
does not fix the merge schedule.  The GPU library also offers a schedule made of synchronous rounds
(every community looks at the same state), which this file restates in plain numpy, integers only,
so that the two can be compared bit for bit:

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
