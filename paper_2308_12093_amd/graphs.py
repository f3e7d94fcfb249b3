"""Device-side graph set-up: chains the preprocessing entry points of the C ABI.

Only sequencing and buffer allocation happen here; self-loops, degrees,
normalisation, the CSR->CSC transpose and the row-index expansion all run in
the library's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _dev_i32(a, device):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def add_self_loops(n, rowptr, col):
    """(rowptr, col) device int32 -> (rowptr', col', deg) with the diagonal present once per row."""
    dev = rowptr.device
    nnz = int(col.numel())
    rowptr_out = torch.empty(n + 1, dtype=torch.int32, device=dev)
    col_out = torch.empty(nnz + n, dtype=torch.int32, device=dev)
    deg = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    ws = B.alloc(B.gnn_scan_workspace_bytes(n), dev)
    nnz2 = B.gnn_add_self_loops_degree(n, nnz, rowptr, col, rowptr_out, col_out, deg, ws)
    return rowptr_out, col_out[:nnz2], deg[:n]


def transpose(n, rowptr, col):
    dev = rowptr.device
    nnz = int(col.numel())
    colptr = torch.empty(n + 1, dtype=torch.int32, device=dev)
    row = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    perm = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    ws = B.alloc(B.gnn_transpose_workspace_bytes(n, nnz), dev)
    B.gnn_csr_transpose(n, nnz, rowptr, col, colptr, row, perm, ws)
    return colptr, row[:nnz], perm[:nnz]


def expand(n, ptr, nnz):
    out = torch.empty(max(nnz, 1), dtype=torch.int32, device=ptr.device)
    B.gnn_expand_ptr(n, nnz, ptr, out)
    return out[:nnz]


def gcn_graph(rowptr_np, col_np, device="cuda", symmetric=True, balanced=True,
              aggregator=B.GNN_AGG_GCN_SYM, eps=0.0) -> B.Graph:
    """Raw pattern (host) -> weighted graph on the device, ready for gcn_layer_fwd / bwd.

    symmetric=True promises an undirected input whose weights are symmetric too, so A' is its
    own transpose and no CSC arrays are built; otherwise the transpose, its values and its
    expanded column index are built as well.  `aggregator` picks the entry values
    (gnn_aggregator_weights); mean weights are never symmetric."""
    n = rowptr_np.size - 1
    rp, c, deg = add_self_loops(n, _dev_i32(rowptr_np, device), _dev_i32(col_np, device))
    nnz = int(c.numel())
    val = torch.empty(max(nnz, 1), dtype=torch.float32, device=device)[:nnz]
    if aggregator == B.GNN_AGG_GCN_SYM:
        B.gnn_gcn_normalize(n, rp, c, deg, val)
    else:
        B.gnn_aggregator_weights(aggregator, eps, n, rp, c, deg, val)
        if aggregator == B.GNN_AGG_MEAN:
            symmetric = False
    erow = expand(n, rp, nnz) if balanced else None
    if symmetric:
        g = B.Graph(n, rp, c, val, erow, symmetric=True)
    else:
        colptr, row, perm = transpose(n, rp, c)
        csc_val = torch.empty_like(val)
        B.gnn_gather_f32(nnz, val, perm, csc_val)
        ecol = expand(n, colptr, nnz) if balanced else None
        g = B.Graph(n, rp, c, val, erow, colptr, row, perm, csc_val, ecol, symmetric=False)
    g.deg = deg
    return g


def gat_graph(rowptr_np, col_np, device="cuda", balanced=True) -> B.Graph:
    """Raw directed pattern (host) -> pattern with self-loops, CSR + CSC + perm on the device."""
    n = rowptr_np.size - 1
    rp, c, deg = add_self_loops(n, _dev_i32(rowptr_np, device), _dev_i32(col_np, device))
    nnz = int(c.numel())
    colptr, row, perm = transpose(n, rp, c)
    erow = expand(n, rp, nnz) if balanced else None
    ecol = expand(n, colptr, nnz) if balanced else None
    g = B.Graph(n, rp, c, None, erow, colptr, row, perm, None, ecol, symmetric=False)
    g.deg = deg
    return g
