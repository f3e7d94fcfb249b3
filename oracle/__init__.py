"""fp64 CPU oracle for the GCN / GAT layer forward and backward passes.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the CPU-baseline leg of the benchmark.  The product path never calls it, and
it shares no code with the HIP library (it does not import the package).

What it computes is the plain definition of each result, once, in one fixed
order, in double precision from inputs widened to double:

* sparse loops (self-loops, degrees, normalisation, CSR->CSC, SpMM, SDDMM and
  the per-edge GAT steps) are the defining loop nests in ``sparse_loops.c``;
* dense products are NumPy's ``@`` on float64 arrays (a library matmul used
  as one step of the definition).

The adaptive reordering and the caching of the paper change the order in
which the same products are taken, not their value (Sec. 3.1), so the oracle
has no notion of "scheme": every scheme of the HIP path is compared with the
same numbers.

Readings of the paper taken here
--------------------------------
* Indices are 0-based: ``rowptr[0] = 0``, ``rowptr[n] = q`` (App. D.1 is 1-based).
* Outputs start from zero (the SpMM listing of App. E.1 accumulates into an
  uninitialised array).
* A' = D^-1/2 (A + I) D^-1/2 with one degree vector, the row sums of the 0/1
  pattern of A + I; an existing diagonal entry is kept, not doubled.
* X' = A' X Theta + 1 b^T with A' indexed [aggregating row][neighbour column]
  (Eq. gcn-fwd); the listing of App. G.1 scatters, i.e. it is this product for
  arrays holding the transposed matrix.
* GAT: the softmax of Eq. gat-fwd-att runs over the stored entries of row i
  (N(i) + {i}); a_src pairs with the row node, a_dst with the column node.
  dL/dX = dL/dM Theta^T (Eq. gat-bwd-features lacks the transpose).
* LeakyReLU' is beta at y <= 0; ReLU' is 0 at 0.
* The ReLU mask of a fused layer is taken from the *given* forward output Y
  (a float32 array), and the LeakyReLU mask optionally from float32 s, d, so
  that both sides of a parity test take each sign decision on identical bits.

parity unpinned: nothing here.  (The SDDMM operational-intensity table of
App. E.2 is not reproduced by any routine; no routine depends on it.)
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparse_loops.c")
_LIB = os.path.join(_HERE, "libgnn_oracle.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the C part with gcc (-O2, OpenMP).  Returns the library path."""
    global _lib
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_add_self_loops_degree.restype = ctypes.c_int64
        _lib.oracle_softmax_xent.restype = ctypes.c_double
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_f64p)


def _opt_f64(a):
    if a is None:
        return None, None
    return _f64(a)


# --------------------------------------------------------------------------
# integer / preprocessing steps
# --------------------------------------------------------------------------
def add_self_loops_degree(rowptr, col):
    """Pattern of A + I and deg (Sec. GCN Forward Pass).  -> rowptr', col', deg (int32)."""
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    n = rowptr.size - 1
    rp2 = np.empty(n + 1, np.int32)
    c2 = np.empty(col.size + n, np.int32)
    deg = np.empty(n, np.int32)
    q2 = _load().oracle_add_self_loops_degree(ctypes.c_int32(n), prp, pc, rp2.ctypes.data_as(_i32p),
                                              c2.ctypes.data_as(_i32p), deg.ctypes.data_as(_i32p))
    return rp2, c2[:q2].copy(), deg


def gcn_normalize(rowptr, col, deg):
    """val_e = 1 / sqrt(deg_i deg_j) for every stored entry of A + I.  -> float64[q]."""
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    deg, pd = _i32(deg)
    val = np.empty(col.size, np.float64)
    _load().oracle_gcn_normalize(ctypes.c_int32(rowptr.size - 1), prp, pc, pd, val.ctypes.data_as(_f64p))
    return val


def aggregator_weights(rowptr, col, deg, kind, eps=0.0):
    """Entry values of the other layers with the same chained product (Sec. 3.1 "Generalizability"):
    "mean": D^-1 (A + I), every entry of row i is 1 / deg_i;  "gin": A + (1 + eps) I."""
    rowptr = np.asarray(rowptr)
    col = np.asarray(col)
    rows = np.repeat(np.arange(rowptr.size - 1), np.diff(rowptr))
    if kind == "mean":
        return 1.0 / np.asarray(deg, np.float64)[rows]
    if kind == "gin":
        return np.where(col == rows, 1.0 + eps, 1.0)
    raise ValueError(kind)


def csr_transpose(rowptr, col):
    """CSC arrays of the same matrix + perm (CSC slot -> CSR slot).  All int32."""
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    n = rowptr.size - 1
    colptr = np.empty(n + 1, np.int32)
    row = np.empty(col.size, np.int32)
    perm = np.empty(col.size, np.int32)
    _load().oracle_csr_transpose(ctypes.c_int32(n), prp, pc, colptr.ctypes.data_as(_i32p),
                                 row.ctypes.data_as(_i32p), perm.ctypes.data_as(_i32p))
    return colptr, row, perm


def is_symmetric(rowptr, col, val) -> bool:
    """A == A^T, pattern and values: the CSC arrays of A equal its CSR arrays entry by entry."""
    colptr, row, perm = csr_transpose(rowptr, col)
    return bool(np.array_equal(colptr, np.asarray(rowptr)) and np.array_equal(row, np.asarray(col))
                and np.array_equal(np.asarray(val)[perm], np.asarray(val)))


# --------------------------------------------------------------------------
# sparse operators
# --------------------------------------------------------------------------
def _sp_call(rowptr, col, val, dense):
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    val, pv = _opt_f64(val)
    dense, pd = _f64(dense)
    n = rowptr.size - 1
    f = dense.shape[1]
    return rowptr, col, val, dense, n, f, prp, pc, pv, pd


def spmm(rowptr, col, val, B):
    """C = A B, A in CSR (App. E.1).  B: [n_cols_of_A, f]."""
    rowptr, col, val, B, n, f, prp, pc, pv, pb = _sp_call(rowptr, col, val, B)
    C = np.empty((n, f), np.float64)
    _load().oracle_spmm(ctypes.c_int32(n), prp, pc, pv, pb, ctypes.c_int32(f), C.ctypes.data_as(_f64p))
    return C


def spmm_transposed(rowptr, col, val, B):
    """C = A^T B for a square A given by its CSR arrays, by scattering (never forms A^T)."""
    rowptr, col, val, B, n, f, prp, pc, pv, pb = _sp_call(rowptr, col, val, B)
    assert B.shape[0] == n
    C = np.empty((n, f), np.float64)
    _load().oracle_spmm_transposed(ctypes.c_int32(n), prp, pc, pv, pb, ctypes.c_int32(f),
                                   C.ctypes.data_as(_f64p))
    return C


def sddmm(rowptr, col, val, B, Ct):
    """D_e = A_e <B_i, Ct_j> on the pattern of A (App. E.2); Ct is the transpose of the paper's C."""
    rowptr, col, val, B, n, f, prp, pc, pv, pb = _sp_call(rowptr, col, val, B)
    Ct, pct = _f64(Ct)
    assert Ct.shape[1] == f
    D = np.empty(col.size, np.float64)
    _load().oracle_sddmm(ctypes.c_int32(n), prp, pc, pv, pb, pct, ctypes.c_int32(f), D.ctypes.data_as(_f64p))
    return D


# --------------------------------------------------------------------------
# GCN layer (Eq. gcn-fwd; Eqs. gcn-bwd-weights / -bias / -x)
# --------------------------------------------------------------------------
def gcn_forward(rowptr, col, val, X, Theta, b=None, relu=False):
    """X' = A' (X Theta) + 1 b^T, optionally followed by ReLU."""
    T = np.asarray(X, np.float64) @ np.asarray(Theta, np.float64)
    Y = spmm(rowptr, col, val, T)
    if b is not None:
        Y = Y + np.asarray(b, np.float64)[None, :]
    if relu:
        Y = np.maximum(Y, 0.0)
    return Y


def gcn_backward(rowptr, col, val, X, Theta, G, Y_relu=None, need_dx=True, symmetric=False):
    """dTheta = X^T A'^T G, db = G^T 1, dX = A'^T G Theta^T.

    ``Y_relu``: the layer's forward output when a ReLU was fused after it; the
    incoming gradient is first multiplied by [Y > 0].
    ``symmetric``: the caller has checked that A' equals its transpose (``is_symmetric``), so
    A'^T G is taken as A' G with the row-gather loop, which is parallel over rows; the scatter
    loop is parallel over feature columns only and takes minutes on the 2^22-node graph."""
    G = np.asarray(G, np.float64)
    if Y_relu is not None:
        G = G * (np.asarray(Y_relu) > 0)
    H = spmm(rowptr, col, val, G) if symmetric else spmm_transposed(rowptr, col, val, G)
    dTheta = np.asarray(X, np.float64).T @ H
    db = G.sum(axis=0)
    dX = H @ np.asarray(Theta, np.float64).T if need_dx else None
    return dTheta, db, dX


def sage_forward(rowptr, col, val, X, W_self, W_neigh, b=None, relu=False):
    """GraphSAGE layer (Sec. 3.1 "Generalizability"): X W_self + A' X W_neigh + 1 b^T, optionally ReLU;
    ``val`` are the entries of the aggregation matrix A' (row-normalised pattern for the mean)."""
    X = np.asarray(X, np.float64)
    Y = X @ np.asarray(W_self, np.float64) + spmm(rowptr, col, val, X) @ np.asarray(W_neigh, np.float64)
    if b is not None:
        Y = Y + np.asarray(b, np.float64)[None, :]
    if relu:
        Y = np.maximum(Y, 0.0)
    return Y


def sage_backward(rowptr, col, val, X, W_self, W_neigh, G, Y_relu=None, need_dx=True):
    """Gradients of sage_forward: dW_self = X^T G, dW_neigh = (A'X)^T G, db = G^T 1,
    dX = G W_self^T + A'^T (G W_neigh^T)."""
    X = np.asarray(X, np.float64)
    G = np.asarray(G, np.float64)
    if Y_relu is not None:
        G = G * (np.asarray(Y_relu) > 0)
    dWs = X.T @ G
    dWn = spmm(rowptr, col, val, X).T @ G
    db = G.sum(axis=0)
    dX = None
    if need_dx:
        dX = G @ np.asarray(W_self, np.float64).T + spmm_transposed(rowptr, col, val, G @ np.asarray(W_neigh, np.float64).T)
    return dWs, dWn, db, dX


def softmax_xent(Z, labels):
    """Sum-reduced softmax cross-entropy and dZ = softmax(Z) - onehot."""
    Z, pz = _f64(Z)
    labels, pl = _i32(labels)
    dZ = np.empty_like(Z)
    loss = _load().oracle_softmax_xent(ctypes.c_int32(Z.shape[0]), ctypes.c_int32(Z.shape[1]), pz, pl,
                                       dZ.ctypes.data_as(_f64p))
    return float(loss), dZ


# --------------------------------------------------------------------------
# GAT layer (Eqs. gat-fwd, gat-fwd-att; Sec. GAT Backward Pass)
# --------------------------------------------------------------------------
def gat_node_attention(M, a_src, a_dst):
    """s_i = <a_src, m_i>, d_i = <a_dst, m_i> per head.  M: [n, h, k]; a_*: [h, k]."""
    M, pm = _f64(M)
    n, h, k = M.shape
    a_src, pas = _f64(a_src)
    a_dst, pad = _f64(a_dst)
    s = np.empty((n, h), np.float64)
    d = np.empty((n, h), np.float64)
    _load().oracle_gat_node_attention(ctypes.c_int32(n), ctypes.c_int32(h), ctypes.c_int32(k), pm, pas, pad,
                                      s.ctypes.data_as(_f64p), d.ctypes.data_as(_f64p))
    return s, d


def gat_edge_softmax(rowptr, col, s, d, slope, decide_fp32=False, tie_eps=0.0, tie_mode=0):
    """alpha = row-softmax(LeakyReLU(s_i + d_j)) and mask = (s_i + d_j > 0), both [q, h]."""
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    s, ps = _f64(s)
    d, pd = _f64(d)
    n, h = s.shape
    alpha = np.empty((col.size, h), np.float64)
    mask = np.empty((col.size, h), np.uint8)
    _load().oracle_gat_edge_softmax(ctypes.c_int32(n), ctypes.c_int32(h), prp, pc, ps, pd,
                                    ctypes.c_double(slope), ctypes.c_int(int(decide_fp32)),
                                    ctypes.c_double(tie_eps), ctypes.c_int(tie_mode),
                                    alpha.ctypes.data_as(_f64p), mask.ctypes.data_as(_u8p))
    return alpha, mask


def gat_aggregate(rowptr, col, alpha, M):
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    alpha, pa = _f64(alpha)
    M, pm = _f64(M)
    n, h, k = M.shape
    Y = np.empty((n, h, k), np.float64)
    _load().oracle_gat_aggregate(ctypes.c_int32(n), ctypes.c_int32(h), ctypes.c_int32(k), prp, pc, pa, pm,
                                 Y.ctypes.data_as(_f64p))
    return Y


def gat_forward(rowptr, col, X, Theta, a_src, a_dst, b, heads, slope, tie_eps=0.0, tie_mode=0):
    """Forward pass; returns a dict with Y [n, h*k] and every intermediate."""
    X = np.asarray(X, np.float64)
    Theta = np.asarray(Theta, np.float64)
    n = X.shape[0]
    hk = Theta.shape[1]
    k = hk // heads
    M = (X @ Theta).reshape(n, heads, k)
    s, d = gat_node_attention(M, np.asarray(a_src).reshape(heads, k), np.asarray(a_dst).reshape(heads, k))
    alpha, mask = gat_edge_softmax(rowptr, col, s, d, slope, False, tie_eps, tie_mode)
    Y = gat_aggregate(rowptr, col, alpha, M).reshape(n, hk)
    if b is not None:
        Y = Y + np.asarray(b, np.float64)[None, :]
    return {"Y": Y, "M": M, "s": s, "d": d, "alpha": alpha, "mask": mask}


def gat_backward_from(rowptr, col, X, Theta, a_src, a_dst, G, M, alpha, mask, slope, need_dx=True):
    """Backward pass from given M, alpha, mask (whatever produced them)."""
    rowptr, prp = _i32(rowptr)
    col, pc = _i32(col)
    M, pm = _f64(M)
    n, h, k = M.shape
    G, pg = _f64(np.asarray(G, np.float64).reshape(n, h, k))
    alpha, pa = _f64(alpha)
    mask = np.ascontiguousarray(mask, np.uint8)
    a_src, pas = _f64(np.asarray(a_src, np.float64).reshape(h, k))
    a_dst, pad = _f64(np.asarray(a_dst, np.float64).reshape(h, k))
    q = col.size
    gy = np.empty((q, h), np.float64)
    ds = np.empty((n, h), np.float64)
    dd = np.empty((n, h), np.float64)
    lib = _load()
    ci = ctypes.c_int32
    lib.oracle_gat_edge_backward(ci(n), ci(h), ci(k), prp, pc, pg, pm, pa, mask.ctypes.data_as(_u8p),
                                 ctypes.c_double(slope), gy.ctypes.data_as(_f64p),
                                 ds.ctypes.data_as(_f64p), dd.ctypes.data_as(_f64p))
    dM = np.empty((n, h, k), np.float64)
    lib.oracle_gat_feature_grad(ci(n), ci(h), ci(k), prp, pc, pa, pg, ds.ctypes.data_as(_f64p),
                                dd.ctypes.data_as(_f64p), pas, pad, dM.ctypes.data_as(_f64p))
    da_src = np.empty((h, k), np.float64)
    da_dst = np.empty((h, k), np.float64)
    lib.oracle_gat_attention_grad(ci(n), ci(h), ci(k), ds.ctypes.data_as(_f64p), pm, da_src.ctypes.data_as(_f64p))
    lib.oracle_gat_attention_grad(ci(n), ci(h), ci(k), dd.ctypes.data_as(_f64p), pm, da_dst.ctypes.data_as(_f64p))
    dM2 = dM.reshape(n, h * k)
    out = {"dW": np.asarray(X, np.float64).T @ dM2, "da_src": da_src, "da_dst": da_dst,
           "db": G.reshape(n, h * k).sum(axis=0), "dM": dM, "ds": ds, "dd": dd, "gy": gy}
    out["dX"] = dM2 @ np.asarray(Theta, np.float64).T if need_dx else None
    return out


def gat_backward(rowptr, col, X, Theta, a_src, a_dst, G, heads, slope, need_dx=True,
                 tie_eps=0.0, tie_mode=0):
    """Backward pass with everything recomputed from the layer inputs."""
    fw = gat_forward(rowptr, col, X, Theta, a_src, a_dst, None, heads, slope, tie_eps, tie_mode)
    return gat_backward_from(rowptr, col, X, Theta, a_src, a_dst, G, fw["M"], fw["alpha"], fw["mask"],
                             slope, need_dx)


def gat_backward_cached(rowptr, col, X, Theta, a_src, a_dst, G, M32, s32, d32, slope, need_dx=True):
    """Backward pass from cached float32 M, s, d: alpha is rebuilt from them in
    double, and every LeakyReLU sign is decided on the float sum s_i + d_j."""
    alpha, mask = gat_edge_softmax(rowptr, col, np.asarray(s32, np.float32), np.asarray(d32, np.float32),
                                   slope, decide_fp32=True)
    return gat_backward_from(rowptr, col, X, Theta, a_src, a_dst, G, np.asarray(M32, np.float32),
                             alpha, mask, slope, need_dx)


# --------------------------------------------------------------------------
# the pieces around the layers in the paper's two-layer GAT network (Sec. 4):
# ELU between the layers, squared-error loss at the end
# --------------------------------------------------------------------------
def elu(x):
    """ELU with alpha = 1: x for x > 0, exp(x) - 1 otherwise."""
    x = np.asarray(x, np.float64)
    return np.where(x > 0.0, x, np.expm1(np.minimum(x, 0.0)))


def elu_grad_from_output(G, Y):
    """G * ELU'(x) written with the output y = ELU(x): ELU'(x) = 1 for x > 0, exp(x) = y + 1 otherwise
    (y > 0 exactly when x > 0).  Y may be a float32 array: its sign is then the decision both
    sides of a comparison share."""
    G = np.asarray(G, np.float64)
    Y = np.asarray(Y)
    return np.where(Y > 0, G, G * (Y.astype(np.float64) + 1.0))


def sum_squared_error(Z, T):
    """loss = 1/2 sum (Z - T)^2 and its gradient Z - T (sum reduction: gradient entries O(1))."""
    E = np.asarray(Z, np.float64) - np.asarray(T, np.float64)
    return 0.5 * float(np.sum(E * E)), E


# --------------------------------------------------------------------------
# the paper's operational-intensity model for SpMM (App. E.1, table)
# --------------------------------------------------------------------------
def csr_to_hybrid(rowptr, col, val, t):
    """ELLPACK / hybrid CSR-COO storage (App. D.3, D.4): the first ``t`` entries of every row go to
    Col, V of width t (kept slot-major, [t][n]; padding: column -1, value 0), the others, row by row, to
    coordinate arrays.  With t >= the longest row the coordinate part is empty and p = t."""
    rowptr, col = np.asarray(rowptr), np.asarray(col)
    n = rowptr.size - 1
    val = np.ones(col.size) if val is None else np.asarray(val, np.float64)
    ell_col = np.full((t, n), -1, np.int32)
    ell_val = np.zeros((t, n), np.float64)
    rows, cols, vals = [], [], []
    for i in range(n):
        r0, r1 = int(rowptr[i]), int(rowptr[i + 1])
        k = min(t, r1 - r0)
        ell_col[:k, i] = col[r0:r0 + k]
        ell_val[:k, i] = val[r0:r0 + k]
        if r1 - r0 > t:
            rows.append(np.full(r1 - r0 - t, i, np.int32))
            cols.append(col[r0 + t:r1])
            vals.append(val[r0 + t:r1])
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt)
    return ell_col, ell_val, cat(rows, np.int32), cat(cols, np.int32), cat(vals, np.float64)


def spmm_ell(ell_col, ell_val, B):
    """C = A B with A in ELLPACK form: row i adds V[i][j] * B[Col[i][j]] over its slots j (padding skipped)."""
    B = np.asarray(B, np.float64)
    t, n = ell_col.shape
    C = np.zeros((n, B.shape[1]))
    for j in range(t):
        live = ell_col[j] >= 0
        C[live] += ell_val[j][live, None] * B[ell_col[j][live]]
    return C


def spmm_coo(n, row, col, val, B):
    """C = A B with A as coordinate triples (App. D.2), in any order, duplicates adding up."""
    B = np.asarray(B, np.float64)
    val = np.ones(len(row)) if val is None else np.asarray(val, np.float64)
    C = np.zeros((n, B.shape[1]))
    np.add.at(C, np.asarray(row), val[:, None] * B[np.asarray(col)])
    return C


def ell_padding_fraction(n: int, q: int, p: int) -> float:
    """Share of zeros in the n x p ELLPACK value matrix of a matrix with q entries (App. E.1)."""
    return 1.0 - q / (n * p)


def spmm_operational_intensity(fmt: str, n: int, q: int, f: int, p: int = 0) -> float:
    """FLOP per byte of C = A B with A n x n (q entries, longest row p), B n x f, 4-byte words.

    FLOPs = 2 q f.  Bytes: the sparse structure once, B once, C read and
    written (the listing accumulates into C)."""
    flops = 2.0 * q * f
    dense = 4.0 * (n * f + 2 * n * f)
    if fmt in ("csr", "csc"):
        sparse = 4.0 * (2 * q + n + 1)
    elif fmt == "coo":
        sparse = 4.0 * 3 * q
    elif fmt == "ellpack":
        sparse = 4.0 * 2 * n * p
    else:
        raise ValueError(fmt)
    return flops / (sparse + dense)
