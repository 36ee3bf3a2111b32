"""Helpers shared by the tests: tiny graph builders, golden-file reader, error metrics."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    """'key v v v' lines -> dict key -> list of token lists (comments skipped)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out.setdefault(k, []).append(v)
    return out


def csr_from_edges(n, edges, self_loops=False):
    """Symmetric CSR (sorted rows) from undirected edge list."""
    adj = [set() for _ in range(n)]
    for a, b in edges:
        if a == b:
            continue
        adj[a].add(b)
        adj[b].add(a)
    if self_loops:
        for i in range(n):
            adj[i].add(i)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    col = []
    for i in range(n):
        col.extend(sorted(adj[i]))
        rowptr[i + 1] = len(col)
    return rowptr, np.asarray(col, dtype=np.int32)


def random_sym_csr(n, p, rng, self_loops=False):
    edges = [(a, b) for a in range(n) for b in range(a + 1, n) if rng.random() < p]
    return csr_from_edges(n, edges, self_loops)


def dense_from_csr(rowptr, colidx, vals=None):
    n = len(rowptr) - 1
    A = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for e in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[e]] += 1.0 if vals is None else float(vals[e])
    return A


def parity_errors(got, ref, abs_ref=None):
    """(normwise error, worst guarded componentwise ratio).

    normwise  = max|got-ref| / max|ref|
    guarded   = max over elements of |got-ref| / (|ref| + abs_ref), where abs_ref is the sum of
                absolute values of the terms of the element's last summation.
    """
    got = np.asarray(got, dtype=np.float64)
    ref64 = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref64)
    denom = np.abs(ref64).max() if ref64.size else 0.0
    normwise = float(diff.max() / denom) if ref64.size and denom > 0 else float(diff.max() if ref64.size else 0.0)
    if abs_ref is None:
        guarded = None
    else:
        scale = np.abs(ref64) + np.asarray(abs_ref, dtype=np.float64)
        ok = scale > 0
        guarded = float((diff[ok] / scale[ok]).max()) if ok.any() else 0.0
        if (~ok).any():
            guarded = max(guarded, float(np.inf) if diff[~ok].max() > 0 else 0.0)
    return normwise, guarded
