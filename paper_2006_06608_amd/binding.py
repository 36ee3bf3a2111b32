"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "GnnError", "lib_path", "load", "exported_symbols",
    "GNN_GCN", "GNN_GIN", "GNN_FLAG_REUSE_PARTITION", "GNN_FLAG_NO_BLOCK_OPT", "GNN_FLAG_XCD_RUNS", "GNN_FLAG_NO_PIPELINE",
    "GNN_FLAG_PIPELINE", "GNN_FLAG_DETERMINISTIC", "GNN_FLAG_FUSION", "GNN_FLAG_ATOMIC_FLUSH", "GNN_FLAG_GCN_NARROW_FIRST", "GNN_FLAG_GCN_UPDATE_FIRST", "GNN_FLAG_NO_FUSION", "GNN_REDUCE_SUM", "GNN_REDUCE_MAX", "GNN_REDUCE_MIN",
    "GNN_REDUCE_MEAN", "gnn_aggregate_reduce", "gnn_aggregate_edge", "gnn_model_workspace_bytes", "gnn_model_forward", "ModelCall", "AggregateCall",
    "gnn_reorder_device", "gnn_apply_perm_csr_device", "gnn_gcn_norm_device", "gnn_aes_device",
    "gnn_bench_stream_read", "gnn_bench_gather_rows", "gnn_csr_transpose_device", "gnn_bench_last_aggregation",
    "gnn_reorder", "gnn_aes", "gnn_gcn_norm", "gnn_apply_perm_csr", "gnn_decide", "gnn_paper_model",
    "gnn_workspace_bytes", "gnn_partition_build", "gnn_workspace_status", "gnn_partition_export",
    "gnn_block_layout_export", "gnn_validate_csr_device", "gnn_aggregate_gcn", "gnn_aggregate_gin", "gnn_aggregate_gin_static",
    "gnn_update_gemm", "gnn_layer_forward", "gnn_layer_forward_timed", "gnn_permute_rows", "gnn_strerror",
    "gnn_version", "alloc_workspace", "gnn_csr_transpose", "gnn_backward_workspace_bytes", "gnn_layer_backward",
]

GNN_GCN, GNN_GIN = 0, 1
GNN_FLAG_REUSE_PARTITION, GNN_FLAG_NO_BLOCK_OPT, GNN_FLAG_XCD_RUNS, GNN_FLAG_NO_PIPELINE = 1, 2, 4, 8
GNN_FLAG_PIPELINE = 16
GNN_FLAG_DETERMINISTIC = 32
GNN_FLAG_FUSION = 64
GNN_FLAG_ATOMIC_FLUSH = 128
GNN_FLAG_GCN_NARROW_FIRST = 256
GNN_FLAG_GCN_UPDATE_FIRST = 1024
GNN_FLAG_NO_FUSION = 512
GNN_REDUCE_SUM, GNN_REDUCE_MAX, GNN_REDUCE_MIN, GNN_REDUCE_MEAN = 0, 1, 2, 3

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("GNN_MI355X_LIB") or os.path.join(_PKG, "libgnn_mi355x.so")

# every symbol include/gnn.h and include/gnn_bench.h declare
_SYMBOLS = [
    "gnn_reorder", "gnn_aes", "gnn_gcn_norm", "gnn_apply_perm_csr", "gnn_decide", "gnn_paper_model",
    "gnn_workspace_bytes", "gnn_partition_build", "gnn_workspace_status", "gnn_partition_export",
    "gnn_block_layout_export", "gnn_validate_csr_device", "gnn_aggregate_gcn", "gnn_aggregate_gin", "gnn_aggregate_gin_static",
    "gnn_aggregate_reduce", "gnn_aggregate_edge", "gnn_model_workspace_bytes", "gnn_model_forward",
    "gnn_update_gemm", "gnn_layer_forward", "gnn_layer_forward_timed", "gnn_permute_rows", "gnn_strerror",
    "gnn_last_hip_error", "gnn_version", "gnn_csr_transpose", "gnn_backward_workspace_bytes", "gnn_layer_backward",
    "gnn_reorder_device", "gnn_apply_perm_csr_device", "gnn_gcn_norm_device", "gnn_aes_device",
    "gnn_bench_stream_read", "gnn_bench_gather_rows", "gnn_csr_transpose_device", "gnn_bench_last_aggregation",
]


class GnnError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {gnn_strerror(code)} (code {code})")
        self.code = code


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def exported_symbols():
    return list(_SYMBOLS)


def load():
    """Load the shared library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2006_06608_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        lib = ctypes.CDLL(_LIB_PATH)
        lib.gnn_workspace_bytes.restype = ctypes.c_size_t
        lib.gnn_backward_workspace_bytes.restype = ctypes.c_size_t
        lib.gnn_model_workspace_bytes.restype = ctypes.c_size_t
        lib.gnn_strerror.restype = ctypes.c_char_p
        for name in _SYMBOLS:
            getattr(lib, name)  # AttributeError if the build lost a symbol
        _lib = lib
    return _lib


# ------------------------------------------------------------------ marshalling helpers
def _i32(x): return ctypes.c_int32(int(x))
def _i64(x): return ctypes.c_int64(int(x))
def _u32(x): return ctypes.c_uint32(int(x))
def _f32(x): return ctypes.c_float(float(x))
def _sz(x): return ctypes.c_size_t(int(x))


def _host(a: Optional[np.ndarray], dtype, name: str):
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: expected a C-contiguous numpy array of {np.dtype(dtype).name}")
    return a.ctypes.data_as(ctypes.c_void_p)


def _dev(t, dtype_name: str, name: str):
    """Device pointer of a contiguous CUDA/HIP torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):  # a raw device address (the static scratch array of gnn_aggregate_gin_static)
        return ctypes.c_void_p(t)
    import torch
    want = {"int32": torch.int32, "float32": torch.float32, "uint8": torch.uint8}[dtype_name]
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != want or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype_name} tensor on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise GnnError(rc, what)


def gnn_strerror(code: int) -> str:
    return load().gnn_strerror(ctypes.c_int(code)).decode()


def gnn_version() -> int:
    return int(load().gnn_version())


# ------------------------------------------------------------------ host-side preparation
def gnn_reorder(rowptr: np.ndarray, colidx: np.ndarray, force: bool = False):
    """-> (perm, iperm, aes, did_reorder)"""
    n = rowptr.size - 1
    perm = np.empty(n, dtype=np.int32)
    iperm = np.empty(n, dtype=np.int32)
    aes = ctypes.c_double(0.0)
    did = ctypes.c_int(0)
    rc = load().gnn_reorder(_i32(n), _host(rowptr, np.int32, "rowptr"), _host(colidx, np.int32, "colidx"),
                            _host(perm, np.int32, "perm"), _host(iperm, np.int32, "iperm"),
                            ctypes.byref(aes), ctypes.byref(did), ctypes.c_int(1 if force else 0))
    _check(rc, "gnn_reorder")
    return perm, iperm, aes.value, bool(did.value)


def gnn_aes(rowptr: np.ndarray, colidx: np.ndarray) -> Tuple[int, float]:
    s = ctypes.c_int64(0)
    a = ctypes.c_double(0.0)
    rc = load().gnn_aes(_i32(rowptr.size - 1), _host(rowptr, np.int32, "rowptr"), _host(colidx, np.int32, "colidx"),
                        ctypes.byref(s), ctypes.byref(a))
    _check(rc, "gnn_aes")
    return int(s.value), float(a.value)


def gnn_gcn_norm(rowptr: np.ndarray, colidx: np.ndarray) -> np.ndarray:
    ew = np.empty(colidx.size, dtype=np.float32)
    rc = load().gnn_gcn_norm(_i32(rowptr.size - 1), _host(rowptr, np.int32, "rowptr"),
                             _host(colidx, np.int32, "colidx"), _host(ew, np.float32, "ew"))
    _check(rc, "gnn_gcn_norm")
    return ew


def gnn_apply_perm_csr(rowptr: np.ndarray, colidx: np.ndarray, perm: np.ndarray, val: Optional[np.ndarray] = None):
    n = rowptr.size - 1
    rp2 = np.empty(n + 1, dtype=np.int32)
    ci2 = np.empty(colidx.size, dtype=np.int32)
    v2 = None if val is None else np.empty(colidx.size, dtype=np.float32)
    rc = load().gnn_apply_perm_csr(_i32(n), _host(rowptr, np.int32, "rowptr"), _host(colidx, np.int32, "colidx"),
                                   _host(val, np.float32, "val"), _host(perm, np.int32, "perm"),
                                   _host(rp2, np.int32, "rowptr2"), _host(ci2, np.int32, "colidx2"),
                                   _host(v2, np.float32, "val2"))
    _check(rc, "gnn_apply_perm_csr")
    return (rp2, ci2) if val is None else (rp2, ci2, v2)


def gnn_csr_transpose(rowptr: np.ndarray, colidx: np.ndarray, val: Optional[np.ndarray] = None):
    n = rowptr.size - 1
    rp2 = np.empty(n + 1, dtype=np.int32)
    ci2 = np.empty(colidx.size, dtype=np.int32)
    v2 = None if val is None else np.empty(colidx.size, dtype=np.float32)
    rc = load().gnn_csr_transpose(_i32(n), _host(rowptr, np.int32, "rowptr"), _host(colidx, np.int32, "colidx"),
                                  _host(val, np.float32, "val"), _host(rp2, np.int32, "rowptr_t"),
                                  _host(ci2, np.int32, "colidx_t"), _host(v2, np.float32, "val_t"))
    _check(rc, "gnn_csr_transpose")
    return (rp2, ci2) if val is None else (rp2, ci2, v2)


def gnn_decide(n: int, nnz: int, max_degree: int, dim: int, ngs: int = 0, dw: int = 0,
               waves_per_block: int = 0) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_int32(ngs), ctypes.c_int32(dw), ctypes.c_int32(waves_per_block)
    rc = load().gnn_decide(_i32(n), _i64(nnz), _i32(max_degree), _i32(dim), ctypes.byref(a), ctypes.byref(b),
                           ctypes.byref(c))
    _check(rc, "gnn_decide")
    return a.value, b.value, c.value


def gnn_paper_model(dim: int, tpw: int, tpb: int, ngs: int) -> Tuple[int, float, int]:
    dw, wpt, smem = ctypes.c_int32(0), ctypes.c_double(0.0), ctypes.c_int64(0)
    rc = load().gnn_paper_model(_i32(dim), _i32(tpw), _i32(tpb), _i32(ngs), ctypes.byref(dw), ctypes.byref(wpt),
                                ctypes.byref(smem))
    _check(rc, "gnn_paper_model")
    return dw.value, wpt.value, smem.value


# ------------------------------------------------------------------ device entry points
def gnn_workspace_bytes(n: int, nnz: int, max_dim: int = 0, ngs: int = 0) -> int:
    return int(load().gnn_workspace_bytes(_i32(n), _i64(nnz), _i32(max_dim), _i32(ngs)))


def alloc_workspace(n: int, nnz: int, max_dim: int = 0, ngs: int = 0, device="cuda"):
    """A uint8 torch tensor of the size gnn_workspace_bytes asks for (torch allocations are 256-byte aligned)."""
    import torch
    nbytes = gnn_workspace_bytes(n, nnz, max_dim, ngs)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _ws(workspace):
    return _dev(workspace, "uint8", "workspace"), _sz(0 if workspace is None else workspace.numel())


def gnn_partition_build(n, nnz, rowptr, ngs, workspace, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_partition_build(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _i32(ngs), wp, wb,
                                    _stream(stream))
    _check(rc, "gnn_partition_build")


def gnn_workspace_status(workspace, stream=None, check: bool = True) -> Tuple[int, int, int]:
    """-> (status code, num_ng, ngs); raises on a non-zero status unless check=False."""
    num = ctypes.c_int64(0)
    ngs = ctypes.c_int32(0)
    rc = load().gnn_workspace_status(_dev(workspace, "uint8", "workspace"), _stream(stream), ctypes.byref(num),
                                     ctypes.byref(ngs))
    if check:
        _check(rc, "gnn_workspace_status")
    return rc, int(num.value), int(ngs.value)


def gnn_partition_export(workspace, stream=None):
    _, num_ng, _ = gnn_workspace_status(workspace, stream)
    node = np.empty(num_ng, dtype=np.int32)
    start = np.empty(num_ng, dtype=np.int32)
    end = np.empty(num_ng, dtype=np.int32)
    rc = load().gnn_partition_export(_dev(workspace, "uint8", "workspace"), _stream(stream), _i64(num_ng),
                                     _host(node, np.int32, "ng_node"), _host(start, np.int32, "ng_start"),
                                     _host(end, np.int32, "ng_end"))
    _check(rc, "gnn_partition_export")
    return node, start, end


def gnn_block_layout_export(workspace, dim: int, dw: int, waves_per_block: int, stream=None):
    """-> (slot int32[num_ng], leader uint8[num_ng], groups_per_block)"""
    _, num_ng, _ = gnn_workspace_status(workspace, stream)
    slot = np.empty(num_ng, dtype=np.int32)
    leader = np.empty(num_ng, dtype=np.uint8)
    gpb = ctypes.c_int32(0)
    rc = load().gnn_block_layout_export(_dev(workspace, "uint8", "workspace"), _stream(stream), _i32(dim), _i32(dw),
                                        _i32(waves_per_block), _i64(num_ng), _host(slot, np.int32, "slot"),
                                        _host(leader, np.uint8, "leader"), ctypes.byref(gpb))
    _check(rc, "gnn_block_layout_export")
    return slot, leader, gpb.value


def gnn_validate_csr_device(n, nnz, rowptr, colidx, stream=None):
    rc = load().gnn_validate_csr_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                        _dev(colidx, "int32", "colidx"), _stream(stream))
    _check(rc, "gnn_validate_csr_device")


def gnn_aggregate_gcn(n, nnz, rowptr, colidx, ew, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0,
                      workspace=None, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_aggregate_gcn(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                                  _dev(ew, "float32", "ew"), _dev(X, "float32", "X"), _dev(out, "float32", "out"),
                                  _i32(dim), _i32(ngs), _i32(dw), _i32(waves_per_block), _u32(flags), wp, wb,
                                  _stream(stream))
    _check(rc, "gnn_aggregate_gcn")


def gnn_aggregate_gin(n, nnz, rowptr, colidx, eps, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0,
                      workspace=None, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_aggregate_gin(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                                  _f32(eps), _dev(X, "float32", "X"), _dev(out, "float32", "out"), _i32(dim),
                                  _i32(ngs), _i32(dw), _i32(waves_per_block), _u32(flags), wp, wb, _stream(stream))
    _check(rc, "gnn_aggregate_gin")


def gnn_aggregate_gin_static(n, nnz, rowptr, colidx, eps, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0,
                             stream=None) -> int:
    """gnn_aggregate_gin on the library's own scratch array (no workspace, nothing allocated); returns the
    device address of that array (accepted by gnn_workspace_status and gnn_partition_export)."""
    addr = ctypes.c_void_p(0)
    rc = load().gnn_aggregate_gin_static(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                         _dev(colidx, "int32", "colidx"), _f32(eps), _dev(X, "float32", "X"),
                                         _dev(out, "float32", "out"), _i32(dim), _i32(ngs), _i32(dw),
                                         _i32(waves_per_block), _u32(flags), _stream(stream), ctypes.byref(addr))
    _check(rc, "gnn_aggregate_gin_static")
    return int(addr.value or 0)


def gnn_bench_last_aggregation() -> str:
    buf = ctypes.create_string_buffer(256)
    _check(load().gnn_bench_last_aggregation(buf, _sz(256)), "gnn_bench_last_aggregation")
    return buf.value.decode()


class AggregateCall:
    """Arguments of gnn_aggregate_gcn (eps None; ew a tensor or None) or gnn_aggregate_gin (eps a number)
    marshalled once, for repeated calls on the same tensors: agg = AggregateCall(...); agg() enqueues one
    aggregation on the stream given here (or on the current one)."""

    def __init__(self, n, nnz, rowptr, colidx, ew, eps, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0,
                 workspace=None, stream=None):
        if eps is not None and ew is not None:
            raise ValueError("GIN aggregation takes no edge weights")
        self._keep = (rowptr, colidx, ew, X, out, workspace)
        wp, wb = _ws(workspace)
        gin = eps is not None
        self._what = "gnn_aggregate_gin" if gin else "gnn_aggregate_gcn"
        self._fn = getattr(load(), self._what)
        self._stream = stream
        self._args = [_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                      _f32(eps) if gin else _dev(ew, "float32", "ew"), _dev(X, "float32", "X"),
                      _dev(out, "float32", "out"), _i32(dim), _i32(ngs), _i32(dw), _i32(waves_per_block), _u32(flags),
                      wp, wb]

    def __call__(self):
        _check(self._fn(*self._args, _stream(self._stream)), self._what)


def gnn_aggregate_reduce(op, n, nnz, rowptr, colidx, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0,
                         workspace=None, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_aggregate_reduce(ctypes.c_int(op), _i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                     _dev(colidx, "int32", "colidx"), _dev(X, "float32", "X"),
                                     _dev(out, "float32", "out"), _i32(dim), _i32(ngs), _i32(dw),
                                     _i32(waves_per_block), _u32(flags), wp, wb, _stream(stream))
    _check(rc, "gnn_aggregate_reduce")


def gnn_aggregate_edge(n, nnz, rowptr, colidx, E, X, out, dim, ngs=0, dw=0, waves_per_block=0, flags=0, workspace=None,
                       stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_aggregate_edge(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                                   _dev(E, "float32", "E"), _dev(X, "float32", "X"), _dev(out, "float32", "out"),
                                   _i32(dim), _i32(ngs), _i32(dw), _i32(waves_per_block), _u32(flags), wp, wb,
                                   _stream(stream))
    _check(rc, "gnn_aggregate_edge")


def gnn_update_gemm(n, K, M, A, W, b, relu, out, stream=None):
    rc = load().gnn_update_gemm(_i32(n), _i32(K), _i32(M), _dev(A, "float32", "A"), _dev(W, "float32", "W"),
                                _dev(b, "float32", "b"), ctypes.c_int(1 if relu else 0), _dev(out, "float32", "out"),
                                _stream(stream))
    _check(rc, "gnn_update_gemm")


def gnn_layer_forward(kind, n, nnz, rowptr, colidx, ew, eps, X, in_dim, W, b, out_dim, relu, out, ngs=0, dw=0,
                      waves_per_block=0, flags=0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_layer_forward(ctypes.c_int(kind), _i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                  _dev(colidx, "int32", "colidx"), _dev(ew, "float32", "ew"), _f32(eps),
                                  _dev(X, "float32", "X"), _i32(in_dim), _dev(W, "float32", "W"),
                                  _dev(b, "float32", "b"), _i32(out_dim), ctypes.c_int(1 if relu else 0),
                                  _dev(out, "float32", "out"), _i32(ngs), _i32(dw), _i32(waves_per_block),
                                  _u32(flags), wp, wb, _stream(stream))
    _check(rc, "gnn_layer_forward")


def _event(ev):
    """hipEvent_t of a recorded-capable torch.cuda.Event (None -> NULL)."""
    if ev is None:
        return None
    if not ev.cuda_event:  # torch creates the handle lazily, on the first record
        raise ValueError("the event has no handle yet: record it once before passing it")
    return ctypes.c_void_p(ev.cuda_event)


def gnn_layer_forward_timed(kind, n, nnz, rowptr, colidx, ew, eps, X, in_dim, W, b, out_dim, relu, out, ngs=0, dw=0,
                            waves_per_block=0, flags=0, workspace=None, stream=None, ev_agg_start=None,
                            ev_agg_stop=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_layer_forward_timed(ctypes.c_int(kind), _i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                        _dev(colidx, "int32", "colidx"), _dev(ew, "float32", "ew"), _f32(eps),
                                        _dev(X, "float32", "X"), _i32(in_dim), _dev(W, "float32", "W"),
                                        _dev(b, "float32", "b"), _i32(out_dim), ctypes.c_int(1 if relu else 0),
                                        _dev(out, "float32", "out"), _i32(ngs), _i32(dw), _i32(waves_per_block),
                                        _u32(flags), wp, wb, _stream(stream), _event(ev_agg_start),
                                        _event(ev_agg_stop))
    _check(rc, "gnn_layer_forward_timed")


def gnn_model_workspace_bytes(n: int, nnz: int, dims: Sequence[int], ngs: int = 0) -> int:
    d = (ctypes.c_int32 * len(dims))(*[int(x) for x in dims])
    return int(load().gnn_model_workspace_bytes(_i32(n), _i64(nnz), _i32(len(dims) - 1), d, _i32(ngs)))


class ModelCall:
    """Arguments of gnn_model_forward marshalled once (pointer arrays, dims), for repeated calls on the
    same tensors: model = ModelCall(...); model() enqueues one forward pass."""

    def __init__(self, kind, n, nnz, rowptr, colidx, ew, eps, X, dims, Ws, bs, out, ngs=0, dw=0, waves_per_block=0,
                 flags=0, workspace=None, stream=None, ev_agg_start=None, ev_agg_stop=None):
        L = len(dims) - 1
        if len(Ws) != L or (bs is not None and len(bs) != L):
            raise ValueError("one weight matrix (and optionally one bias) per layer")
        self._keep = (rowptr, colidx, ew, X, list(Ws), None if bs is None else list(bs), out, workspace)
        ptr_array = ctypes.c_void_p * L
        self._dims = (ctypes.c_int32 * (L + 1))(*[int(x) for x in dims])
        self._W = ptr_array(*[_dev(W, "float32", "W").value for W in Ws])
        self._b = None if bs is None else ptr_array(*[None if b is None else _dev(b, "float32", "b").value for b in bs])
        ev = lambda evs: None if evs is None else ptr_array(*[None if e is None else _event(e).value for e in evs])
        self._ev0, self._ev1 = ev(ev_agg_start), ev(ev_agg_stop)
        wp, wb = _ws(workspace)
        self._fn = load().gnn_model_forward
        self._stream = stream
        self._args = [ctypes.c_int(kind), _i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                      _dev(colidx, "int32", "colidx"), _dev(ew, "float32", "ew"), _f32(eps), _dev(X, "float32", "X"),
                      _i32(L), self._dims, self._W, self._b, _dev(out, "float32", "out"), _i32(ngs), _i32(dw),
                      _i32(waves_per_block), _u32(flags), wp, wb]

    def __call__(self, flags=None):
        args = self._args if flags is None else self._args[:16] + [_u32(flags)] + self._args[17:]
        rc = self._fn(*args, _stream(self._stream), self._ev0, self._ev1)
        _check(rc, "gnn_model_forward")


def gnn_model_forward(kind, n, nnz, rowptr, colidx, ew, eps, X, dims, Ws, bs, out, ngs=0, dw=0, waves_per_block=0,
                      flags=0, workspace=None, stream=None, ev_agg_start=None, ev_agg_stop=None):
    ModelCall(kind, n, nnz, rowptr, colidx, ew, eps, X, dims, Ws, bs, out, ngs, dw, waves_per_block, flags, workspace,
              stream, ev_agg_start, ev_agg_stop)()


def gnn_backward_workspace_bytes(n: int, nnz: int, in_dim: int, out_dim: int, ngs: int = 0) -> int:
    return int(load().gnn_backward_workspace_bytes(_i32(n), _i64(nnz), _i32(in_dim), _i32(out_dim), _i32(ngs)))


def gnn_layer_backward(kind, n, nnz, rowptr_t, colidx_t, ew_t, eps, P, in_dim, W, out_dim, relu, Y, dY, dX, dW, db,
                       ngs=0, dw=0, waves_per_block=0, flags=0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    rc = load().gnn_layer_backward(ctypes.c_int(kind), _i32(n), _i64(nnz), _dev(rowptr_t, "int32", "rowptr_t"),
                                   _dev(colidx_t, "int32", "colidx_t"), _dev(ew_t, "float32", "ew_t"), _f32(eps),
                                   _dev(P, "float32", "P"), _i32(in_dim), _dev(W, "float32", "W"), _i32(out_dim),
                                   ctypes.c_int(1 if relu else 0), _dev(Y, "float32", "Y"), _dev(dY, "float32", "dY"),
                                   _dev(dX, "float32", "dX"), _dev(dW, "float32", "dW"), _dev(db, "float32", "db"),
                                   _i32(ngs), _i32(dw), _i32(waves_per_block), _u32(flags), wp, wb, _stream(stream))
    _check(rc, "gnn_layer_backward")


def gnn_permute_rows(n, dim, perm, X, Y, stream=None):
    rc = load().gnn_permute_rows(_i32(n), _i32(dim), _dev(perm, "int32", "perm"), _dev(X, "float32", "X"),
                                 _dev(Y, "float32", "Y"), _stream(stream))
    _check(rc, "gnn_permute_rows")


# ------------------------------------------------------------------ graph preparation on the device
def gnn_reorder_device(n, nnz, rowptr, colidx, max_rounds: int = 64, stream=None):
    """Round-based community renumbering on DEVICE int32 tensors.  Returns (perm, iperm, rounds)."""
    import torch
    perm = torch.empty(max(int(n), 1), dtype=torch.int32, device=rowptr.device)[: int(n)]
    iperm = torch.empty(max(int(n), 1), dtype=torch.int32, device=rowptr.device)[: int(n)]
    rounds = ctypes.c_int32(0)
    rc = load().gnn_reorder_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                                   _dev(perm, "int32", "perm"), _dev(iperm, "int32", "iperm"), _i32(max_rounds),
                                   ctypes.byref(rounds), _stream(stream))
    _check(rc, "gnn_reorder_device")
    return perm, iperm, int(rounds.value)


def gnn_apply_perm_csr_device(n, nnz, rowptr, colidx, perm, val=None, stream=None):
    """gnn_apply_perm_csr on DEVICE tensors.  Returns (rowptr2, colidx2) or (rowptr2, colidx2, val2)."""
    import torch
    rowptr2 = torch.empty(int(n) + 1, dtype=torch.int32, device=rowptr.device)
    colidx2 = torch.empty(max(int(nnz), 1), dtype=torch.int32, device=rowptr.device)[: int(nnz)]
    val2 = None if val is None else torch.empty(max(int(nnz), 1), dtype=torch.float32, device=rowptr.device)[: int(nnz)]
    rc = load().gnn_apply_perm_csr_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                          _dev(colidx, "int32", "colidx"), _dev(val, "float32", "val"),
                                          _dev(perm, "int32", "perm"), _dev(rowptr2, "int32", "rowptr2"),
                                          _dev(colidx2, "int32", "colidx2"), _dev(val2, "float32", "val2"),
                                          _stream(stream))
    _check(rc, "gnn_apply_perm_csr_device")
    return (rowptr2, colidx2) if val is None else (rowptr2, colidx2, val2)


def gnn_gcn_norm_device(n, nnz, rowptr, colidx, stream=None):
    """Eq. 2 weights on DEVICE tensors; returns the float32 tensor ew[nnz] (work is only enqueued)."""
    import torch
    ew = torch.empty(max(int(nnz), 1), dtype=torch.float32, device=rowptr.device)[: int(nnz)]
    rc = load().gnn_gcn_norm_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                                    _dev(ew, "float32", "ew"), _stream(stream))
    _check(rc, "gnn_gcn_norm_device")
    return ew


def gnn_aes_device(n, nnz, rowptr, colidx, stream=None):
    """Eq. 4 on DEVICE tensors.  Returns (aes_sum, aes, should_reorder)."""
    total, mean, want = ctypes.c_int64(0), ctypes.c_double(0.0), ctypes.c_int(0)
    rc = load().gnn_aes_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"), _dev(colidx, "int32", "colidx"),
                               ctypes.byref(total), ctypes.byref(mean), ctypes.byref(want), _stream(stream))
    _check(rc, "gnn_aes_device")
    return int(total.value), float(mean.value), bool(want.value)


# ------------------------------------------------------------------ measuring kernels
def gnn_bench_stream_read(src, sink, stream=None):
    """Enqueues one sequential read of the whole float32 DEVICE tensor src (sink: float32 DEVICE tensor, 1 element)."""
    rc = load().gnn_bench_stream_read(_dev(src, "float32", "src"), _sz(src.numel() * 4), _dev(sink, "float32", "sink"),
                                      _stream(stream))
    _check(rc, "gnn_bench_stream_read")


def gnn_bench_gather_rows(n, dim, X, idx, sink, stream=None):
    """Enqueues a bare gather of the rows idx (int32 DEVICE tensor) of X[n, dim]."""
    rc = load().gnn_bench_gather_rows(_i32(n), _i32(dim), _dev(X, "float32", "X"), _dev(idx, "int32", "idx"),
                                      _i64(idx.numel()), _dev(sink, "float32", "sink"), _stream(stream))
    _check(rc, "gnn_bench_gather_rows")


def gnn_csr_transpose_device(n, nnz, rowptr, colidx, val=None, stream=None):
    """gnn_csr_transpose on DEVICE tensors.  Returns (rowptr_t, colidx_t) or (rowptr_t, colidx_t, val_t)."""
    import torch
    rowptr_t = torch.empty(int(n) + 1, dtype=torch.int32, device=rowptr.device)
    colidx_t = torch.empty(max(int(nnz), 1), dtype=torch.int32, device=rowptr.device)[: int(nnz)]
    val_t = None if val is None else torch.empty(max(int(nnz), 1), dtype=torch.float32, device=rowptr.device)[: int(nnz)]
    rc = load().gnn_csr_transpose_device(_i32(n), _i64(nnz), _dev(rowptr, "int32", "rowptr"),
                                         _dev(colidx, "int32", "colidx"), _dev(val, "float32", "val"),
                                         _dev(rowptr_t, "int32", "rowptr_t"), _dev(colidx_t, "int32", "colidx_t"),
                                         _dev(val_t, "float32", "val_t"), _stream(stream))
    _check(rc, "gnn_csr_transpose_device")
    return (rowptr_t, colidx_t) if val is None else (rowptr_t, colidx_t, val_t)
