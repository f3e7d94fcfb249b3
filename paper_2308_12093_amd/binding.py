"""ctypes binding of ``libgnn_mi355x.so`` (the C ABI declared in ``include/gnn.h``).

Argument marshalling only: every function below has the name of the C entry
point it calls and passes device pointers taken from torch tensors
(``tensor.data_ptr()``) plus the current torch HIP stream.  No arithmetic of
the method happens in Python.  There is no CPU fallback: importing this
module raises if the library has not been built.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgnn_mi355x.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2308_12093_amd.build` "
        "(the HIP library is required; there is no fallback path)")

lib = ctypes.CDLL(LIB_PATH)

# ---- enums -------------------------------------------------------------------
GNN_OK = 0
(GNN_ERR_INVALID_ARG, GNN_ERR_BAD_GRAPH, GNN_ERR_BUFFER_TOO_SMALL, GNN_ERR_STATE,
 GNN_ERR_UNSUPPORTED, GNN_ERR_HIP) = range(1, 7)
GNN_LAYER_GCN, GNN_LAYER_GAT, GNN_LAYER_SAGE = 0, 1, 2
GNN_ORDER_AUTO, GNN_ORDER_TRANSFORM_FIRST, GNN_ORDER_PROPAGATE_FIRST = 0, 1, 2
GNN_BWD_AUTO, GNN_BWD_FUSED_PROPAGATE, GNN_BWD_SPLIT_PROPAGATE = 0, 1, 2
(GNN_CACHE_AUTO, GNN_CACHE_NONE, GNN_CACHE_AX, GNN_CACHE_GAT_FEAT, GNN_CACHE_GAT_FEAT_NODEATT,
 GNN_CACHE_GAT_FEAT_EDGE) = range(6)
GNN_SELECT_PAPER_RULE, GNN_SELECT_CALIBRATED = 0, 1
GNN_AGG_GCN_SYM, GNN_AGG_MEAN, GNN_AGG_GIN_SUM = 0, 1, 2

_vp = ctypes.c_void_p
_i32 = ctypes.c_int32
_i64 = ctypes.c_int64
_sz = ctypes.c_size_t


class gnn_graph_t(ctypes.Structure):
    _fields_ = [("n", _i32), ("nnz", _i32),
                ("csr_rowptr", _vp), ("csr_col", _vp), ("csr_val", _vp), ("csr_erow", _vp),
                ("csc_colptr", _vp), ("csc_row", _vp), ("csc_perm", _vp), ("csc_val", _vp), ("csc_ecol", _vp),
                ("symmetric", _i32)]


class gnn_plan_desc_t(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_int), ("n", _i32), ("nnz", _i32), ("f_in", _i32), ("f_out", _i32),
                ("heads", _i32), ("need_input_grad", _i32), ("has_bias", _i32), ("fuse_relu", _i32),
                ("leaky_slope", ctypes.c_float), ("order", ctypes.c_int), ("bwd", ctypes.c_int),
                ("cache", ctypes.c_int), ("selection", ctypes.c_int), ("constant_input", _i32), ("fuse_elu", _i32)]


class gnn_plan_info_t(ctypes.Structure):
    _fields_ = [("order", ctypes.c_int), ("bwd", ctypes.c_int), ("cache", ctypes.c_int),
                ("cache_bytes", _sz), ("workspace_bytes", _sz),
                ("transient_fwd", _i64), ("transient_bwd", _i64),
                ("spmm_width_fwd", _i64), ("spmm_width_bwd", _i64)]


_BUFS = [_vp, _sz, _vp, _sz, _vp]
# every symbol the header declares, with its prototype
_PROTOS = {
    "gnn_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "gnn_plan_create": (ctypes.c_int, [ctypes.POINTER(gnn_plan_desc_t), ctypes.POINTER(_vp)]),
    "gnn_plan_query": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_plan_info_t)]),
    "gnn_plan_destroy": (None, [_vp]),
    "gnn_plan_reset_cache": (ctypes.c_int, [_vp]),
    "gnn_spmm_time_model_us": (ctypes.c_double, [_i64, _i64, _i32]),
    # layer calls end with (cache, cache_bytes, workspace, workspace_bytes, hip_stream)
    "gcn_layer_fwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 4 + _BUFS),
    "gcn_layer_bwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 7 + _BUFS),
    "sage_layer_fwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 5 + _BUFS),
    "sage_layer_bwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 9 + _BUFS),
    "gat_layer_fwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 6 + _BUFS),
    "gat_layer_bwd": (ctypes.c_int, [_vp, ctypes.POINTER(gnn_graph_t)] + [_vp] * 11 + _BUFS),
    "gnn_add_self_loops_degree": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_i32), _vp, _sz, _vp]),
    "gnn_scan_workspace_bytes": (_sz, [_i32]),
    "gnn_gcn_normalize": (ctypes.c_int, [_i32, _vp, _vp, _vp, _vp, _vp]),
    "gnn_aggregator_weights": (ctypes.c_int, [ctypes.c_int, ctypes.c_float, _i32, _vp, _vp, _vp, _vp, _vp]),
    "gnn_hyb_workspace_bytes": (_sz, [_i32]),
    "gnn_csr_hyb_count": (ctypes.c_int, [_i32, _vp, _i32, _vp, ctypes.POINTER(_i32), ctypes.POINTER(_i32), _vp, _sz, _vp]),
    "gnn_csr_to_hyb": (ctypes.c_int, [_i32, _i32] + [_vp] * 10),
    "gnn_spmm_ell": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _i32, _vp, _vp]),
    "gnn_spmm_coo": (ctypes.c_int, [_i32, _i64, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp]),
    "gnn_spmm_hyb": (ctypes.c_int, [_i32, _i32, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "gnn_csr_transpose": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "gnn_transpose_workspace_bytes": (_sz, [_i32, _i32]),
    "gnn_expand_ptr": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp]),
    "gnn_gather_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "gnn_spmm_csr": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _sz, _vp]),
    "gnn_spmm_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "gnn_spmm_csr_static": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp]),
    "gnn_gat_aggregate_csr": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, ctypes.c_float, _vp,
                                             _i32, _vp, _vp, _vp, _sz, _vp]),
    "gnn_gat_aggregate_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "gnn_sddmm_csr": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "gnn_gemm": (ctypes.c_int, [_i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]),
    "gnn_gemm_workspace_bytes": (_sz, [_i32, _i32, _i64, _i64, _i64]),
    "gnn_softmax_xent": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "gnn_sum_squared_error": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
}
EXPORTS = tuple(_PROTOS)
for _name, (_res, _args) in _PROTOS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


class GnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.gnn_status_string(status).decode()} (status {status})")


def _check(status: int, where: str):
    if status != GNN_OK:
        raise GnnError(status, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _bufs(cache, workspace):
    """(cache, cache_bytes, workspace, workspace_bytes, stream): the tail of every layer call."""
    return _ptr(cache), _nbytes(cache), _ptr(workspace), _nbytes(workspace), _stream()


def alloc(nbytes: int, device="cuda"):
    """A 256-byte aligned device buffer of at least ``nbytes`` bytes (torch owns the memory)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---- graph -------------------------------------------------------------------
class Graph:
    """Holds the device tensors of a graph and the ``gnn_graph_t`` pointing at them."""

    def __init__(self, n, rowptr, col, val=None, erow=None, colptr=None, row=None, perm=None,
                 csc_val=None, ecol=None, symmetric=False):
        self.tensors = dict(rowptr=rowptr, col=col, val=val, erow=erow, colptr=colptr, row=row, perm=perm,
                            csc_val=csc_val, ecol=ecol)
        self.n = int(n)
        self.nnz = int(col.numel())
        self.c = gnn_graph_t(self.n, self.nnz, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(erow),
                             _ptr(colptr), _ptr(row), _ptr(perm), _ptr(csc_val), _ptr(ecol), int(bool(symmetric)))

    def __getattr__(self, name):
        t = self.__dict__.get("tensors", {})
        if name in t:
            return t[name]
        raise AttributeError(name)


# ---- plan --------------------------------------------------------------------
class Plan:
    def __init__(self, layer, n, nnz, f_in, f_out, heads=1, need_input_grad=True, has_bias=False,
                 fuse_relu=False, leaky_slope=0.2, order=GNN_ORDER_AUTO, bwd=GNN_BWD_AUTO, cache=GNN_CACHE_AUTO,
                 selection=GNN_SELECT_PAPER_RULE, constant_input=False, fuse_elu=False):
        self.desc = gnn_plan_desc_t(layer, n, nnz, f_in, f_out, heads, int(need_input_grad), int(has_bias),
                                    int(fuse_relu), leaky_slope, order, bwd, cache, selection,
                                    int(constant_input), int(fuse_elu))
        self.handle = _vp()
        _check(gnn_plan_create(self.desc, self.handle), "gnn_plan_create")
        self.info = gnn_plan_query(self.handle)

    def reset_cache(self):
        _check(lib.gnn_plan_reset_cache(self.handle), "gnn_plan_reset_cache")

    def close(self):
        if self.handle:
            lib.gnn_plan_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gnn_plan_create(desc: gnn_plan_desc_t, out_handle) -> int:
    return lib.gnn_plan_create(ctypes.byref(desc), ctypes.byref(out_handle))


def gnn_plan_query(handle) -> gnn_plan_info_t:
    info = gnn_plan_info_t()
    _check(lib.gnn_plan_query(handle, ctypes.byref(info)), "gnn_plan_query")
    return info


def gnn_status_string(status: int) -> str:
    return lib.gnn_status_string(status).decode()


# ---- layers --------------------------------------------------------------------
def gcn_layer_fwd(plan: Plan, graph: Graph, X, W, b, Y, cache, workspace):
    _check(lib.gcn_layer_fwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W), _ptr(b), _ptr(Y),
                             *_bufs(cache, workspace)), "gcn_layer_fwd")


def gcn_layer_bwd(plan: Plan, graph: Graph, X, W, Y, dY, dW, db, dX, cache, workspace):
    _check(lib.gcn_layer_bwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W), _ptr(Y), _ptr(dY), _ptr(dW),
                             _ptr(db), _ptr(dX), *_bufs(cache, workspace)), "gcn_layer_bwd")


def sage_layer_fwd(plan: Plan, graph: Graph, X, W_self, W_neigh, b, Y, cache, workspace):
    _check(lib.sage_layer_fwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W_self), _ptr(W_neigh), _ptr(b),
                              _ptr(Y), *_bufs(cache, workspace)), "sage_layer_fwd")


def sage_layer_bwd(plan: Plan, graph: Graph, X, W_self, W_neigh, Y, dY, dW_self, dW_neigh, db, dX, cache, workspace):
    _check(lib.sage_layer_bwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W_self), _ptr(W_neigh), _ptr(Y),
                              _ptr(dY), _ptr(dW_self), _ptr(dW_neigh), _ptr(db), _ptr(dX), *_bufs(cache, workspace)), "sage_layer_bwd")


def gat_layer_fwd(plan: Plan, graph: Graph, X, W, a_src, a_dst, b, Y, cache, workspace):
    _check(lib.gat_layer_fwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W), _ptr(a_src), _ptr(a_dst),
                             _ptr(b), _ptr(Y), *_bufs(cache, workspace)), "gat_layer_fwd")


def gat_layer_bwd(plan: Plan, graph: Graph, X, W, a_src, a_dst, dY, dW, da_src, da_dst, db, dX, cache, workspace,
                  Y=None):
    _check(lib.gat_layer_bwd(plan.handle, ctypes.byref(graph.c), _ptr(X), _ptr(W), _ptr(a_src), _ptr(a_dst),
                             _ptr(Y), _ptr(dY), _ptr(dW), _ptr(da_src), _ptr(da_dst), _ptr(db), _ptr(dX),
                             *_bufs(cache, workspace)), "gat_layer_bwd")


# ---- preprocessing ---------------------------------------------------------------
def gnn_scan_workspace_bytes(n):
    return lib.gnn_scan_workspace_bytes(n)


def gnn_add_self_loops_degree(n, nnz, rowptr, col, rowptr_out, col_out, deg_out, workspace) -> int:
    out = _i32(0)
    _check(lib.gnn_add_self_loops_degree(n, nnz, _ptr(rowptr), _ptr(col), _ptr(rowptr_out), _ptr(col_out),
                                         _ptr(deg_out), ctypes.byref(out), _ptr(workspace), _nbytes(workspace),
                                         _stream()), "gnn_add_self_loops_degree")
    return out.value


def gnn_gcn_normalize(n, rowptr, col, deg, val_out):
    _check(lib.gnn_gcn_normalize(n, _ptr(rowptr), _ptr(col), _ptr(deg), _ptr(val_out), _stream()),
           "gnn_gcn_normalize")


def gnn_aggregator_weights(kind, eps, n, rowptr, col, deg, val_out):
    _check(lib.gnn_aggregator_weights(int(kind), float(eps), n, _ptr(rowptr), _ptr(col), _ptr(deg), _ptr(val_out),
                                      _stream()), "gnn_aggregator_weights")


def gnn_transpose_workspace_bytes(n, nnz):
    return lib.gnn_transpose_workspace_bytes(n, nnz)


def gnn_csr_transpose(n, nnz, rowptr, col, colptr_out, row_out, perm_out, workspace):
    _check(lib.gnn_csr_transpose(n, nnz, _ptr(rowptr), _ptr(col), _ptr(colptr_out), _ptr(row_out), _ptr(perm_out),
                                 _ptr(workspace), _nbytes(workspace), _stream()), "gnn_csr_transpose")


def gnn_expand_ptr(n, nnz, ptr, out):
    _check(lib.gnn_expand_ptr(n, nnz, _ptr(ptr), _ptr(out), _stream()), "gnn_expand_ptr")


def gnn_gather_f32(count, src, perm, out):
    _check(lib.gnn_gather_f32(count, _ptr(src), _ptr(perm), _ptr(out), _stream()), "gnn_gather_f32")


def gnn_spmm_time_model_us(n, nnz, f) -> float:
    return float(lib.gnn_spmm_time_model_us(n, nnz, f))


# ---- operators ----------------------------------------------------------------------
def gnn_spmm_workspace_bytes(n, nnz, f):
    return lib.gnn_spmm_workspace_bytes(n, nnz, f)


def gnn_spmm_csr(n, nnz, rowptr, col, val, erow, B, f, C, bias=None, relu=False, workspace=None):
    _check(lib.gnn_spmm_csr(n, nnz, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(erow), _ptr(B), f, _ptr(C),
                            _ptr(bias), int(relu), _ptr(workspace), _nbytes(workspace), _stream()), "gnn_spmm_csr")


GNN_STATIC_SCRATCH_BYTES = 32 << 20


def gnn_spmm_csr_static(n, nnz, rowptr, col, val, erow, B, f, C, bias=None, relu=False):
    _check(lib.gnn_spmm_csr_static(n, nnz, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(erow), _ptr(B), f, _ptr(C),
                                   _ptr(bias), int(relu), _stream()), "gnn_spmm_csr_static")


# ---- other storage formats (format comparison) --------------------------------------
def gnn_hyb_workspace_bytes(n):
    return lib.gnn_hyb_workspace_bytes(n)


def gnn_csr_hyb_count(n, rowptr, t, rest_ptr_out, workspace):
    """Returns (rest_nnz, longest_row)."""
    rest, longest = _i32(0), _i32(0)
    _check(lib.gnn_csr_hyb_count(n, _ptr(rowptr), t, _ptr(rest_ptr_out), ctypes.byref(rest), ctypes.byref(longest),
                                 _ptr(workspace), _nbytes(workspace), _stream()), "gnn_csr_hyb_count")
    return rest.value, longest.value


def gnn_csr_to_hyb(n, t, rowptr, col, val, rest_ptr, ell_col, ell_val, coo_row, coo_col, coo_val):
    _check(lib.gnn_csr_to_hyb(n, t, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(rest_ptr), _ptr(ell_col), _ptr(ell_val),
                              _ptr(coo_row), _ptr(coo_col), _ptr(coo_val), _stream()), "gnn_csr_to_hyb")


def gnn_spmm_ell(n, t, ell_col, ell_val, B, f, C):
    _check(lib.gnn_spmm_ell(n, t, _ptr(ell_col), _ptr(ell_val), _ptr(B), f, _ptr(C), _stream()), "gnn_spmm_ell")


def gnn_spmm_coo(n, nnz, row, col, val, B, f, C, accumulate=False):
    _check(lib.gnn_spmm_coo(n, nnz, _ptr(row), _ptr(col), _ptr(val), _ptr(B), f, _ptr(C), int(accumulate),
                            _stream()), "gnn_spmm_coo")


def gnn_spmm_hyb(n, t, ell_col, ell_val, rest_nnz, coo_row, coo_col, coo_val, B, f, C):
    _check(lib.gnn_spmm_hyb(n, t, _ptr(ell_col), _ptr(ell_val), rest_nnz, _ptr(coo_row), _ptr(coo_col),
                            _ptr(coo_val), _ptr(B), f, _ptr(C), _stream()), "gnn_spmm_hyb")


def gnn_sddmm_csr(n, nnz, erow, col, val, B, Ct, heads, f, D):
    _check(lib.gnn_sddmm_csr(n, nnz, _ptr(erow), _ptr(col), _ptr(val), _ptr(B), _ptr(Ct), heads, f, _ptr(D),
                             _stream()), "gnn_sddmm_csr")


def gnn_gat_aggregate_workspace_bytes(nnz, heads, f):
    return lib.gnn_gat_aggregate_workspace_bytes(nnz, heads, f)


def gnn_gat_aggregate_csr(n, nnz, rowptr, erow, col, M, s, d, heads, f, leaky_slope, bias, elu, Y, stat_out, workspace):
    _check(lib.gnn_gat_aggregate_csr(n, nnz, _ptr(rowptr), _ptr(erow), _ptr(col), _ptr(M), _ptr(s), _ptr(d), heads, f,
                                     float(leaky_slope), _ptr(bias), int(elu), _ptr(Y), _ptr(stat_out), _ptr(workspace),
                                     _nbytes(workspace), _stream()), "gnn_gat_aggregate_csr")


def gnn_gemm_workspace_bytes(trans_a, trans_b, M, N, K):
    return lib.gnn_gemm_workspace_bytes(int(trans_a), int(trans_b), M, N, K)


def gnn_gemm(trans_a, trans_b, M, N, K, A, B, C, bias=None, relu=False, workspace=None):
    _check(lib.gnn_gemm(int(trans_a), int(trans_b), M, N, K, _ptr(A), _ptr(B), _ptr(C), _ptr(bias), int(relu),
                        _ptr(workspace), _nbytes(workspace), _stream()), "gnn_gemm")


def gnn_sum_squared_error(count, Z, T, dZ, loss_out, workspace):
    _check(lib.gnn_sum_squared_error(count, _ptr(Z), _ptr(T), _ptr(dZ), _ptr(loss_out), _ptr(workspace),
                                     _nbytes(workspace), _stream()), "gnn_sum_squared_error")


def gnn_softmax_xent(n, c, Z, labels, dZ, loss_out, workspace):
    _check(lib.gnn_softmax_xent(n, c, _ptr(Z), _ptr(labels), _ptr(dZ), _ptr(loss_out), _ptr(workspace),
                                _nbytes(workspace), _stream()), "gnn_softmax_xent")
