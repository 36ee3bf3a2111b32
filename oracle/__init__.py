"""CPU oracle for the GNN aggregation path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``gnn_oracle.c`` plus the layer/model compositions.  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the GPU library never does, and this package never imports the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .parallel_reorder import parallel_reorder, parallel_reorder_numpy  # noqa: F401  (round-based renumbering)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnn_oracle.c")
_LIB = os.path.join(_HERE, "libgnn_oracle.so")


def build(force: bool = False) -> str:
    """Compile gnn_oracle.c with gcc -O2 (no OpenMP, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_aes_sum.restype = ctypes.c_int64
        _lib.orc_ng_partition.restype = ctypes.c_int64
        _lib.orc_eq5_wpt.restype = ctypes.c_double
        _lib.orc_eq5_smem.restype = ctypes.c_int64
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# ------------------------------------------------------------------ operations
def aggregate_gcn(rowptr, colidx, ew, X, want_abs: bool = False):
    """Eq. 2 aggregation: out = (CSR with weights ew) @ X.  ew None = unit weights."""
    rowptr, colidx, X = _i32(rowptr), _i32(colidx), _f32(X)
    ew = None if ew is None else _f32(ew)
    n, dim = rowptr.size - 1, X.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    ab = np.empty((n, dim), dtype=np.float64) if want_abs else None
    _L().orc_aggregate_gcn(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(ew), _p(X), ctypes.c_int32(dim),
                           _p(out), _p(ab))
    return (out, ab) if want_abs else out


def aggregate_edge_vec(rowptr, colidx, E, X, want_abs: bool = False):
    """Aggregation with a feature vector per stored entry (Sec. 3.1): out_i = sum_e E[e,:] * X[colidx[e],:]
    elementwise, E float32 [nnz, dim] in CSR order."""
    rowptr, colidx, X, E = _i32(rowptr), _i32(colidx), _f32(X), _f32(E)
    n, dim = rowptr.size - 1, X.shape[1]
    assert E.shape == (colidx.size, dim)
    out = np.empty((n, dim), dtype=np.float32)
    ab = np.empty((n, dim), dtype=np.float64) if want_abs else None
    _L().orc_aggregate_edge_vec(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(E), _p(X), ctypes.c_int32(dim),
                                _p(out), _p(ab))
    return (out, ab) if want_abs else out


def aggregate_gin(rowptr, colidx, eps: float, X, want_abs: bool = False):
    """Eq. 3 aggregation: out_i = (1+eps) x_i + sum_{j in N(i)} x_j."""
    rowptr, colidx, X = _i32(rowptr), _i32(colidx), _f32(X)
    n, dim = rowptr.size - 1, X.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    ab = np.empty((n, dim), dtype=np.float64) if want_abs else None
    _L().orc_aggregate_gin(ctypes.c_int32(n), _p(rowptr), _p(colidx), ctypes.c_float(eps), _p(X),
                           ctypes.c_int32(dim), _p(out), _p(ab))
    return (out, ab) if want_abs else out


REDUCE_MAX, REDUCE_MIN, REDUCE_MEAN = 1, 2, 3


def aggregate_reduce(rowptr, colidx, X, op: int, want_abs: bool = False):
    """Sec. 3.1 aggregations over the neighbour embeddings alone: max, min or mean per feature;
    rows without entries give 0."""
    assert op in (REDUCE_MAX, REDUCE_MIN, REDUCE_MEAN)
    rowptr, colidx, X = _i32(rowptr), _i32(colidx), _f32(X)
    n, dim = rowptr.size - 1, X.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    ab = np.empty((n, dim), dtype=np.float64) if want_abs else None
    _L().orc_aggregate_reduce(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(X), ctypes.c_int32(dim),
                              ctypes.c_int32(op), _p(out), _p(ab))
    return (out, ab) if want_abs else out


def gemm_bias_act(A, W, b=None, relu: bool = False, want_abs: bool = False):
    """Update phase: act(A @ W + b)."""
    A, W = _f32(A), _f32(W)
    b = None if b is None else _f32(b)
    n, K = A.shape
    M = W.shape[1]
    assert W.shape[0] == K
    out = np.empty((n, M), dtype=np.float32)
    ab = np.empty((n, M), dtype=np.float64) if want_abs else None
    _L().orc_gemm_bias_act(ctypes.c_int32(n), ctypes.c_int32(K), ctypes.c_int32(M), _p(A), _p(W), _p(b),
                           ctypes.c_int32(1 if relu else 0), _p(out), _p(ab))
    return (out, ab) if want_abs else out


def bias_act(Z, b=None, relu: bool = False):
    Z = _f32(Z)
    b = None if b is None else _f32(b)
    out = np.empty_like(Z)
    _L().orc_bias_act(ctypes.c_int32(Z.shape[0]), ctypes.c_int32(Z.shape[1]), _p(Z), _p(b),
                      ctypes.c_int32(1 if relu else 0), _p(out))
    return out


def gcn_norm(rowptr, colidx) -> np.ndarray:
    """Eq. 2 weights 1/sqrt(d_i d_j), d = stored row length."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    ew = np.empty(colidx.size, dtype=np.float32)
    _L().orc_gcn_norm(ctypes.c_int32(rowptr.size - 1), _p(rowptr), _p(colidx), _p(ew))
    return ew


def aes_sum(rowptr, colidx) -> int:
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    return int(_L().orc_aes_sum(ctypes.c_int32(rowptr.size - 1), _p(rowptr), _p(colidx)))


def aes(rowptr, colidx) -> float:
    """Eq. 4."""
    nnz = int(rowptr[-1])
    return aes_sum(rowptr, colidx) / nnz if nnz else 0.0


def aes_threshold(n: int) -> int:
    return int(_L().orc_aes_threshold(ctypes.c_int32(n)))


def should_reorder(rowptr, colidx) -> bool:
    n = len(rowptr) - 1
    return bool(_L().orc_should_reorder(ctypes.c_int32(n), ctypes.c_int64(int(rowptr[-1])),
                                        ctypes.c_int64(aes_sum(rowptr, colidx))))


def ng_partition(rowptr, ngs: int):
    """Sec. 4.1 neighbor groups: arrays (node, start, end), half-open CSR ranges."""
    rowptr = _i32(rowptr)
    n = rowptr.size - 1
    cnt = int(_L().orc_ng_partition(ctypes.c_int32(n), _p(rowptr), ctypes.c_int32(ngs), None, None, None))
    node = np.empty(cnt, dtype=np.int32)
    start = np.empty(cnt, dtype=np.int32)
    end = np.empty(cnt, dtype=np.int32)
    _L().orc_ng_partition(ctypes.c_int32(n), _p(rowptr), ctypes.c_int32(ngs), _p(node), _p(start), _p(end))
    return node, start, end


def alg1_layout(ng_node, warp_per_block: int, dim: int):
    """Algorithm 1: per neighbor group (slot index, float offset of the slot, leader flag)."""
    ng_node = _i32(ng_node)
    k = ng_node.size
    slot = np.empty(k, dtype=np.int32)
    addr = np.empty(k, dtype=np.int64)
    leader = np.empty(k, dtype=np.uint8)
    _L().orc_alg1_layout(ctypes.c_int64(k), _p(ng_node), ctypes.c_int32(warp_per_block), ctypes.c_int32(dim),
                         _p(slot), _p(addr), _p(leader))
    return slot, addr, leader


def eq5_wpt(ngs: int, dim: int, dw: int) -> float:
    return float(_L().orc_eq5_wpt(ctypes.c_int32(ngs), ctypes.c_int32(dim), ctypes.c_int32(dw)))


def eq5_smem(tpb: int, tpw: int, dim: int) -> int:
    return int(_L().orc_eq5_smem(ctypes.c_int32(tpb), ctypes.c_int32(tpw), ctypes.c_int32(dim)))


def eq6_dw(dim: int, tpw: int) -> int:
    return int(_L().orc_eq6_dw(ctypes.c_int32(dim), ctypes.c_int32(tpw)))


def reorder(rowptr, colidx) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 5.1 renumbering (always applied): perm[old] = new, iperm[new] = old."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.size - 1
    perm = np.empty(n, dtype=np.int32)
    iperm = np.empty(n, dtype=np.int32)
    rc = _L().orc_reorder(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(perm), _p(iperm))
    assert rc == 0
    return perm, iperm


def apply_perm_csr(rowptr, colidx, perm, val=None):
    rowptr, colidx, perm = _i32(rowptr), _i32(colidx), _i32(perm)
    val = None if val is None else _f32(val)
    n = rowptr.size - 1
    rp2 = np.empty(n + 1, dtype=np.int32)
    ci2 = np.empty(colidx.size, dtype=np.int32)
    v2 = None if val is None else np.empty(colidx.size, dtype=np.float32)
    _L().orc_apply_perm_csr(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(val), _p(perm), _p(rp2), _p(ci2), _p(v2))
    return (rp2, ci2) if val is None else (rp2, ci2, v2)


def permute_rows(X, perm) -> np.ndarray:
    X, perm = _f32(X), _i32(perm)
    Y = np.empty_like(X)
    _L().orc_permute_rows(ctypes.c_int32(X.shape[0]), ctypes.c_int32(X.shape[1]), _p(perm), _p(X), _p(Y))
    return Y


# ------------------------------------------------------------------ layers and models
# Order inside a layer follows Sec. 3.1: GCN reduces the dimension first (Update, then
# Aggregation); GIN aggregates at full dimension, then updates.  Values between operations
# are stored as float.
def _aggregate_f64(rowptr, colidx, w64, X64):
    """sum_e w[e] * X[col_e,:] in double, nothing rounded to float (error scales only)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    X64 = np.ascontiguousarray(X64, dtype=np.float64)
    w64 = None if w64 is None else np.ascontiguousarray(w64, dtype=np.float64)
    n, dim = rowptr.size - 1, X64.shape[1]
    out = np.empty((n, dim), dtype=np.float64)
    _L().orc_aggregate_f64(ctypes.c_int32(n), _p(rowptr), _p(colidx), _p(w64), _p(X64), ctypes.c_int32(dim), _p(out))
    return out


def gcn_layer(rowptr, colidx, ew, X, W, b=None, relu: bool = False, want_abs=False):
    """act(A_hat (X W) + b).  want_abs=True adds the layer's error scale |A_hat| (|X| |W|) + |b|: the sum
    of absolute values of all terms of both operations, in double throughout, against which a
    floating-point evaluation in any order is judged.  want_abs="both" adds, third, the stricter scale
    of the last operation alone, |A_hat| |fl(X W)| + |b| (fl = the product as stored in float)."""
    if not want_abs:
        H = gemm_bias_act(X, W, None, False)
        return bias_act(aggregate_gcn(rowptr, colidx, ew, H), b, relu)
    H, Habs = gemm_bias_act(X, W, None, False, want_abs=True)
    Z, Zabs = aggregate_gcn(rowptr, colidx, ew, H, want_abs=True)
    babs = 0.0 if b is None else np.abs(_f32(b)).astype(np.float64)
    scale = _aggregate_f64(rowptr, colidx, None if ew is None else np.abs(_f32(ew)).astype(np.float64), Habs) + babs
    out = bias_act(Z, b, relu)
    return (out, scale, Zabs + babs) if want_abs == "both" else (out, scale)


def gin_layer(rowptr, colidx, eps, X, W, b=None, relu: bool = False, want_abs=False):
    """act(((1+eps) X + sum_N X) W + b).  want_abs=True adds the layer's error scale
    (|1+eps| |X| + sum_N |X|) |W| + |b|, in double throughout; want_abs="both" adds, third, the stricter
    scale of the last operation alone, |fl(aggregate)| |W| + |b|."""
    if not want_abs:
        return gemm_bias_act(aggregate_gin(rowptr, colidx, eps, X), W, b, relu)
    A, Aabs = aggregate_gin(rowptr, colidx, eps, X, want_abs=True)
    out, last = gemm_bias_act(A, W, b, relu, want_abs=True)
    babs = 0.0 if b is None else np.abs(_f32(b)).astype(np.float64)
    scale = Aabs @ np.abs(_f32(W)).astype(np.float64) + babs
    return (out, scale, last) if want_abs == "both" else (out, scale)


def gcn_model(rowptr, colidx, ew, X, Ws: Sequence[np.ndarray], bs: Optional[Sequence] = None,
              want_abs: bool = False):
    """ReLU after every layer but the last."""
    H = X
    ab = None
    for l, W in enumerate(Ws):
        last = l == len(Ws) - 1
        b = None if bs is None else bs[l]
        if last and want_abs:
            H, ab = gcn_layer(rowptr, colidx, ew, H, W, b, relu=False, want_abs=True)
        else:
            H = gcn_layer(rowptr, colidx, ew, H, W, b, relu=not last)
    return (H, ab) if want_abs else H


def gin_model(rowptr, colidx, eps, X, Ws: Sequence[np.ndarray], bs: Optional[Sequence] = None,
              want_abs: bool = False):
    H = X
    ab = None
    for l, W in enumerate(Ws):
        last = l == len(Ws) - 1
        b = None if bs is None else bs[l]
        if last and want_abs:
            H, ab = gin_layer(rowptr, colidx, eps, H, W, b, relu=False, want_abs=True)
        else:
            H = gin_layer(rowptr, colidx, eps, H, W, b, relu=not last)
    return (H, ab) if want_abs else H


# ------------------------------------------------------------------ the same loops on several cores
# For the benchmark's all-cores baseline only.  Rows of an aggregation and of the dense layer are
# independent, so disjoint row ranges (balanced by their number of entries) of the very same C loops
# are handed to threads (ctypes releases the interpreter lock during a call).  Results equal the
# single-thread functions bit for bit (tests/test_oracle_layers.py).
def _row_ranges(rowptr, parts: int):
    n = rowptr.size - 1
    cost = rowptr.astype(np.int64) + np.arange(n + 1, dtype=np.int64)  # entries + one unit per row
    cuts = np.searchsorted(cost, np.linspace(0, cost[-1], parts + 1)[1:-1])
    edges = [0] + [int(c) for c in cuts] + [n]
    return [(a, b) for a, b in zip(edges[:-1], edges[1:]) if b > a]


def _run_threads(fn, ranges, threads):
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(lambda r: fn(*r), ranges))


def _off(a: np.ndarray, row: int):
    return ctypes.c_void_p(a.ctypes.data + row * a.strides[0])


def gin_layer_threads(rowptr, colidx, eps, X, W, b, relu: bool, threads: int):
    rowptr, colidx, X, W = _i32(rowptr), _i32(colidx), _f32(X), _f32(W)
    b = None if b is None else _f32(b)
    n, K, M = rowptr.size - 1, X.shape[1], W.shape[1]
    A = np.empty((n, K), dtype=np.float32)
    out = np.empty((n, M), dtype=np.float32)
    L = _L()

    def work(r0, r1):
        L.orc_aggregate_gin_rows(ctypes.c_int32(r0), ctypes.c_int32(r1), _p(rowptr), _p(colidx), ctypes.c_float(eps),
                                 _p(X), ctypes.c_int32(K), _p(A), None)
        L.orc_gemm_bias_act(ctypes.c_int32(r1 - r0), ctypes.c_int32(K), ctypes.c_int32(M), _off(A, r0), _p(W), _p(b),
                            ctypes.c_int32(1 if relu else 0), _off(out, r0), None)

    _run_threads(work, _row_ranges(rowptr, 4 * threads), threads)
    return out


def gcn_layer_threads(rowptr, colidx, ew, X, W, b, relu: bool, threads: int):
    rowptr, colidx, X, W = _i32(rowptr), _i32(colidx), _f32(X), _f32(W)
    ew = None if ew is None else _f32(ew)
    b = None if b is None else _f32(b)
    n, K, M = rowptr.size - 1, X.shape[1], W.shape[1]
    H = np.empty((n, M), dtype=np.float32)
    Z = np.empty((n, M), dtype=np.float32)
    out = np.empty((n, M), dtype=np.float32)
    L = _L()
    ranges = _row_ranges(rowptr, 4 * threads)
    _run_threads(lambda r0, r1: L.orc_gemm_bias_act(ctypes.c_int32(r1 - r0), ctypes.c_int32(K), ctypes.c_int32(M),
                                                    _off(X, r0), _p(W), None, ctypes.c_int32(0), _off(H, r0), None),
                 ranges, threads)

    def work(r0, r1):  # rowptr + r0 keeps absolute positions, so colidx and ew are passed whole
        L.orc_aggregate_gcn(ctypes.c_int32(r1 - r0), _off(rowptr, r0), _p(colidx), _p(ew), _p(H), ctypes.c_int32(M),
                            _off(Z, r0), None)
        L.orc_bias_act(ctypes.c_int32(r1 - r0), ctypes.c_int32(M), _off(Z, r0), _p(b), ctypes.c_int32(1 if relu else 0),
                       _off(out, r0))

    _run_threads(work, ranges, threads)
    return out


def aggregate_gcn_threads(rowptr, colidx, ew, X, threads: int):
    rowptr, colidx, X = _i32(rowptr), _i32(colidx), _f32(X)
    ew = None if ew is None else _f32(ew)
    n, dim = rowptr.size - 1, X.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    L = _L()
    _run_threads(lambda r0, r1: L.orc_aggregate_gcn(ctypes.c_int32(r1 - r0), _off(rowptr, r0), _p(colidx), _p(ew), _p(X),
                                                    ctypes.c_int32(dim), _off(out, r0), None),
                 _row_ranges(rowptr, 4 * threads), threads)
    return out


# ------------------------------------------------------------------ backward pass (training)
# Gradients of the layers above, by the chain rule, each product accumulated in double and stored
# as float between operations (as the forward pass does).  The aggregation of gradients runs over
# the transposed graph: d/dX of (A X) applied to G is A^T G.
def csr_transpose(rowptr, colidx, val=None):
    """Entry (i, j, v) -> (j, i, v); rows of the result sorted by column (stable counting order)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.size - 1
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    order = np.argsort(colidx, kind="stable")  # ties keep ascending row order
    rp_t = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(colidx, minlength=n), out=rp_t[1:])
    ci_t = rows[order].astype(np.int32)
    if val is None:
        return rp_t.astype(np.int32), ci_t
    return rp_t.astype(np.int32), ci_t, _f32(val)[order]


def _mm64(A, B):
    return (np.asarray(A, dtype=np.float64) @ np.asarray(B, dtype=np.float64))


def gcn_layer_backward(rowptr, colidx, ew, X, W, relu, Y, dY, want_abs: bool = False):
    """Forward Y = act(A_hat (X W) + b).  Returns dX, dW, db (and their error scales)."""
    X, W, dY = _f32(X), _f32(W), _f32(dY)
    dZ = np.where(_f32(Y) > 0, dY, np.float32(0)) if relu else dY
    db = dZ.astype(np.float64).sum(axis=0).astype(np.float32)
    rp_t, ci_t, ew_t = csr_transpose(rowptr, colidx, _f32(ew))
    dH, dH_abs = aggregate_gcn(rp_t, ci_t, ew_t, dZ, want_abs=True)
    dW = _mm64(X.T, dH).astype(np.float32)
    dX = _mm64(dH, W.T).astype(np.float32)
    if not want_abs:
        return dX, dW, db
    s_dW = _mm64(np.abs(X).T, dH_abs)
    s_dX = _mm64(dH_abs, np.abs(W).T)
    s_db = np.abs(dZ).astype(np.float64).sum(axis=0)
    return (dX, dW, db), (s_dX, s_dW, s_db)


def gin_layer_backward(rowptr, colidx, eps, A, W, relu, Y, dY, want_abs: bool = False):
    """Forward Y = act(A W + b) with A = (1+eps) X + sum_N X (A is the saved aggregation).
    Returns dX, dW, db (and their error scales)."""
    A, W, dY = _f32(A), _f32(W), _f32(dY)
    dZ = np.where(_f32(Y) > 0, dY, np.float32(0)) if relu else dY
    db = dZ.astype(np.float64).sum(axis=0).astype(np.float32)
    dW = _mm64(A.T, dZ).astype(np.float32)
    dA64 = _mm64(dZ, W.T)
    dA = dA64.astype(np.float32)
    rp_t, ci_t = csr_transpose(rowptr, colidx)
    if not want_abs:
        return aggregate_gin(rp_t, ci_t, eps, dA), dW, db
    dX, _ = aggregate_gin(rp_t, ci_t, eps, dA, want_abs=True)
    dA_abs = _mm64(np.abs(dZ), np.abs(W).T).astype(np.float32)
    _, s_dX = aggregate_gin(rp_t, ci_t, abs(1.0 + eps) - 1.0, dA_abs, want_abs=True)
    s_dW = _mm64(np.abs(A).T, np.abs(dZ))
    s_db = np.abs(dZ).astype(np.float64).sum(axis=0)
    return (dX, dW, db), (s_dX, s_dW, s_db)
