"""Pins for the fp64 oracle: it is checked against things other than itself.

* dense brute force written here from the equations (GCN fwd/bwd, SDDMM);
* library routines (scipy sparse product and transpose, torch fp64 autograd
  on dense masked-softmax attention, torch cross-entropy);
* central finite differences of a scalar loss;
* closed forms and invariants (complete graph, zero attention vector, slope 1,
  identical heads, one node, softmax rows sum to 1, adjoint identity);
* numbers the paper prints (SpMM operational intensities, App. E.1 table).
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from paper_2308_12093_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_graph(n=37, q=160, seed=3, diagonal=True):
    rng = np.random.default_rng(seed)
    return synth.random_directed_graph(n, q, rng, allow_diagonal=diagonal)


def dense_pattern(rowptr, col):
    n = rowptr.size - 1
    A = np.zeros((n, n))
    for i in range(n):
        A[i, col[rowptr[i]:rowptr[i + 1]]] = 1.0
    return A


# ------------------------------------------------------------------ S1, S2
def test_self_loops_and_degree_against_dense():
    rowptr, col = small_graph(diagonal=True)          # some rows already hold their diagonal
    A = dense_pattern(rowptr, col)
    assert A.diagonal().sum() > 0 and A.diagonal().sum() < A.shape[0]
    rp2, c2, deg = oracle.add_self_loops_degree(rowptr, col)
    Ahat = np.minimum(A + np.eye(A.shape[0]), 1.0)    # diagonal set, never doubled
    np.testing.assert_array_equal(dense_pattern(rp2, c2), Ahat)
    np.testing.assert_array_equal(deg, Ahat.sum(axis=1).astype(np.int32))
    for i in range(A.shape[0]):                       # ascending, no duplicates
        r = c2[rp2[i]:rp2[i + 1]]
        assert np.all(np.diff(r) > 0)
    assert rp2[0] == 0 and rp2[-1] == c2.size


def test_self_loops_empty_rows_and_empty_graph():
    rowptr = np.zeros(6, np.int32)
    rp2, c2, deg = oracle.add_self_loops_degree(rowptr, np.zeros(0, np.int32))
    np.testing.assert_array_equal(rp2, np.arange(6))
    np.testing.assert_array_equal(c2, np.arange(5))
    np.testing.assert_array_equal(deg, np.ones(5))


def test_normalisation_against_dense_formula():
    rowptr, col = small_graph()
    rp2, c2, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp2, c2, deg)
    Ahat = dense_pattern(rp2, c2)
    Dm = np.diag(Ahat.sum(axis=1) ** -0.5)
    Aprime = Dm @ Ahat @ Dm
    got = sp.csr_matrix((val, c2, rp2), shape=Ahat.shape).toarray()
    np.testing.assert_allclose(got, Aprime, rtol=1e-14, atol=0)


def test_complete_graph_normalises_to_uniform():
    n = 9
    rowptr = np.arange(n + 1, dtype=np.int32) * (n - 1)
    col = np.concatenate([[j for j in range(n) if j != i] for i in range(n)]).astype(np.int32)
    rp2, c2, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp2, c2, deg)
    np.testing.assert_allclose(val, 1.0 / n, rtol=1e-15)
    rng = np.random.default_rng(0)
    X, W = rng.standard_normal((n, 5)), rng.standard_normal((5, 3))
    Y = oracle.gcn_forward(rp2, c2, val, X, W)
    np.testing.assert_allclose(Y, np.tile((X @ W).mean(axis=0), (n, 1)), rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------------ S3
def test_transpose_against_scipy_and_perm_semantics():
    rowptr, col = small_graph(n=53, q=400, seed=5)
    q = col.size
    colptr, row, perm = oracle.csr_transpose(rowptr, col)
    A = sp.csr_matrix((np.arange(1, q + 1, dtype=np.float64), col, rowptr), shape=(53, 53))
    At = A.T.tocsr()
    At.sort_indices()
    np.testing.assert_array_equal(colptr, At.indptr)
    np.testing.assert_array_equal(row, At.indices)
    np.testing.assert_array_equal(perm, At.data.astype(np.int64) - 1)   # data carried the CSR slot
    assert sorted(perm.tolist()) == list(range(q))
    for j in range(53):
        assert np.all(np.diff(row[colptr[j]:colptr[j + 1]]) > 0)


# ------------------------------------------------------------------ S5, SDDMM
def test_spmm_against_scipy_and_dense():
    rowptr, col = small_graph(n=41, q=300, seed=7)
    rng = np.random.default_rng(1)
    val = rng.standard_normal(col.size)
    B = rng.standard_normal((41, 13))
    A = sp.csr_matrix((val, col, rowptr), shape=(41, 41))
    np.testing.assert_allclose(oracle.spmm(rowptr, col, val, B), A @ B, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm_transposed(rowptr, col, val, B), A.T @ B, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm(rowptr, col, None, B), dense_pattern(rowptr, col) @ B,
                               rtol=1e-13, atol=1e-13)


def test_adjoint_identity_on_directed_graph():
    rowptr, col = small_graph(n=64, q=500, seed=11)
    assert (dense_pattern(rowptr, col) != dense_pattern(rowptr, col).T).any()
    rng = np.random.default_rng(2)
    val = rng.standard_normal(col.size)
    X, G = rng.standard_normal((64, 6)), rng.standard_normal((64, 6))
    lhs = np.sum(oracle.spmm(rowptr, col, val, X) * G)
    rhs = np.sum(X * oracle.spmm_transposed(rowptr, col, val, G))
    assert abs(lhs - rhs) <= 1e-12 * (1 + abs(lhs))
    # and through the CSC arrays: A^T as a CSR matrix is (colptr, row, val[perm])
    colptr, row, perm = oracle.csr_transpose(rowptr, col)
    np.testing.assert_allclose(oracle.spmm(colptr, row, val[perm], G),
                               oracle.spmm_transposed(rowptr, col, val, G), rtol=1e-12, atol=1e-13)


def test_sddmm_against_dense():
    rowptr, col = small_graph(n=29, q=200, seed=13)
    rng = np.random.default_rng(3)
    val = rng.standard_normal(col.size)
    B, Ct = rng.standard_normal((29, 7)), rng.standard_normal((29, 7))
    full = B @ Ct.T
    rows = np.repeat(np.arange(29), np.diff(rowptr))
    np.testing.assert_allclose(oracle.sddmm(rowptr, col, val, B, Ct), val * full[rows, col], rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------------ GCN layer
def _gcn_case(seed=0, n=33, m=6, k=4, directed=True):
    rng = np.random.default_rng(seed)
    rowptr, col = small_graph(n=n, q=5 * n, seed=seed + 100, diagonal=False)
    rp2, c2, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp2, c2, deg)
    X, W = rng.standard_normal((n, m)), rng.standard_normal((m, k))
    b, G = rng.standard_normal(k), rng.standard_normal((n, k))
    return rp2, c2, val, X, W, b, G


def test_gcn_forward_backward_against_dense_brute_force():
    rp, c, val, X, W, b, G = _gcn_case()
    n = X.shape[0]
    Ahat = dense_pattern(rp, c)
    Dm = np.diag(Ahat.sum(axis=1) ** -0.5)
    Ap = Dm @ Ahat @ Dm
    np.testing.assert_allclose(oracle.gcn_forward(rp, c, val, X, W, b), Ap @ X @ W + b, rtol=1e-12, atol=1e-13)
    dW, db, dX = oracle.gcn_backward(rp, c, val, X, W, G)
    np.testing.assert_allclose(dW, X.T @ Ap.T @ G, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, G.T @ np.ones(n), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dX, Ap.T @ G @ W.T, rtol=1e-12, atol=1e-13)


def test_symmetric_shortcut_of_the_backward_pass():
    """gcn_backward(symmetric=True) replaces A'^T G by A' G: equal to the scatter form exactly when A' is
    symmetric, which is_symmetric must tell apart from a directed graph."""
    rng = np.random.default_rng(5)
    n = 40
    r, c = rng.integers(0, n, 150), rng.integers(0, n, 150)
    rowptr, col = synth.coo_to_csr(n, np.concatenate([r, c]), np.concatenate([c, r]))      # undirected
    rp, cc, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, cc, deg)
    assert oracle.is_symmetric(rp, cc, val)
    X, W, G = rng.standard_normal((n, 6)), rng.standard_normal((6, 4)), rng.standard_normal((n, 4))
    a, b = oracle.gcn_backward(rp, cc, val, X, W, G), oracle.gcn_backward(rp, cc, val, X, W, G, symmetric=True)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-13)
    drp, dcol = synth.coo_to_csr(n, r, c)                                                  # directed
    drp, dcol, ddeg = oracle.add_self_loops_degree(drp, dcol)
    assert not oracle.is_symmetric(drp, dcol, oracle.gcn_normalize(drp, dcol, ddeg))
    mean = oracle.aggregator_weights(rp, cc, deg, "mean")                                  # symmetric pattern, not values
    assert not oracle.is_symmetric(rp, cc, mean)


def test_gcn_orderings_agree():
    """(A'X)Theta == A'(X Theta); X^T(A'^T G) == (A'X)^T G; (A'^T G)Theta^T == A'^T(G Theta^T)."""
    rp, c, val, X, W, b, G = _gcn_case(seed=4)
    Y = oracle.gcn_forward(rp, c, val, X, W)
    P = oracle.spmm(rp, c, val, X)
    np.testing.assert_allclose(P @ W, Y, rtol=1e-12, atol=1e-13)
    dW, _, dX = oracle.gcn_backward(rp, c, val, X, W, G)
    np.testing.assert_allclose(P.T @ G, dW, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm_transposed(rp, c, val, G @ W.T), dX, rtol=1e-12, atol=1e-13)


def test_gcn_backward_against_torch_autograd_with_relu():
    rp, c, val, X, W, b, G = _gcn_case(seed=5)
    Ap = torch.tensor(sp.csr_matrix((val, c, rp), shape=(X.shape[0],) * 2).toarray())
    Xt, Wt, bt = (torch.tensor(a, requires_grad=True) for a in (X, W, b))
    Y = torch.relu(Ap @ Xt @ Wt + bt)
    (Y * torch.tensor(G)).sum().backward()
    Yo = oracle.gcn_forward(rp, c, val, X, W, b, relu=True)
    np.testing.assert_allclose(Yo, Y.detach().numpy(), rtol=1e-12, atol=1e-13)
    dW, db, dX = oracle.gcn_backward(rp, c, val, X, W, G, Y_relu=Yo)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_gcn_single_node():
    rp, c, deg = oracle.add_self_loops_degree(np.zeros(2, np.int32), np.zeros(0, np.int32))
    val = oracle.gcn_normalize(rp, c, deg)
    X, W, b = np.array([[1.0, -2.0]]), np.array([[0.5], [3.0]]), np.array([0.25])
    np.testing.assert_allclose(oracle.gcn_forward(rp, c, val, X, W, b), X @ W + b)


# ------------------------------------------------------------------ GAT layer
def _gat_case(seed=0, n=31, m=5, h=3, k=4):
    rng = np.random.default_rng(seed)
    rowptr, col = small_graph(n=n, q=4 * n, seed=seed + 200, diagonal=False)
    rp, c, _ = oracle.add_self_loops_degree(rowptr, col)
    X, W = rng.standard_normal((n, m)), rng.standard_normal((m, h * k)) * 0.7
    a_src, a_dst = rng.standard_normal((h, k)), rng.standard_normal((h, k))
    b, G = rng.standard_normal(h * k), rng.standard_normal((n, h * k))
    return rp, c, X, W, a_src, a_dst, b, G, h, k


def _torch_dense_gat(rp, c, X, W, a_src, a_dst, b, h, k, slope):
    """Dense masked-softmax attention written directly from Eq. gat-fwd-att, per head."""
    n = X.shape[0]
    pat = torch.tensor(dense_pattern(rp, c)) > 0
    outs = []
    for p in range(h):
        Mp = X @ W[:, p * k:(p + 1) * k]                         # n x k
        e = torch.empty(n, n, dtype=torch.float64)
        cat_i = Mp @ a_src[p]                                    # a^T [m_i || m_j] = a_src.m_i + a_dst.m_j
        cat_j = Mp @ a_dst[p]
        e = torch.nn.functional.leaky_relu(cat_i[:, None] + cat_j[None, :], slope)
        e = e.masked_fill(~pat, float("-inf"))
        alpha = torch.softmax(e, dim=1)
        outs.append(alpha @ Mp + b[p * k:(p + 1) * k])
    return torch.cat(outs, dim=1)


def test_gat_forward_backward_against_torch_autograd():
    slope = 0.2
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case()
    tens = [torch.tensor(a, requires_grad=True) for a in (X, W, a_src, a_dst, b)]
    Y = _torch_dense_gat(rp, c, *tens, h, k, slope)
    (Y * torch.tensor(G)).sum().backward()
    fw = oracle.gat_forward(rp, c, X, W, a_src, a_dst, b, h, slope)
    np.testing.assert_allclose(fw["Y"], Y.detach().numpy(), rtol=1e-11, atol=1e-12)
    bw = oracle.gat_backward(rp, c, X, W, a_src, a_dst, G, h, slope)
    for name, t in zip(("dX", "dW", "da_src", "da_dst", "db"), tens):
        np.testing.assert_allclose(bw[name], t.grad.numpy(), rtol=1e-10, atol=1e-11, err_msg=name)


def test_gat_backward_against_finite_differences():
    slope = 0.2
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=9, n=17, m=4, h=2, k=3)
    bw = oracle.gat_backward(rp, c, X, W, a_src, a_dst, G, h, slope)

    def loss(X_, W_, as_, ad_, b_):
        return float(np.sum(oracle.gat_forward(rp, c, X_, W_, as_, ad_, b_, h, slope)["Y"] * G))

    args = [X, W, a_src, a_dst, b]
    rng = np.random.default_rng(0)
    for idx, name in enumerate(("dX", "dW", "da_src", "da_dst", "db")):
        base = args[idx]
        for _ in range(6):
            pos = tuple(rng.integers(0, s) for s in base.shape)
            step = 1e-6
            hi, lo = base.copy(), base.copy()
            hi[pos] += step
            lo[pos] -= step
            fd = (loss(*[hi if t == idx else a for t, a in enumerate(args)])
                  - loss(*[lo if t == idx else a for t, a in enumerate(args)])) / (2 * step)
            ref = bw[name].reshape(base.shape)[pos]
            assert abs(fd - ref) <= 1e-6 * (1 + abs(ref)), (name, pos, fd, ref)


def test_gcn_backward_against_finite_differences():
    rp, c, val, X, W, b, G = _gcn_case(seed=8, n=15, m=4, k=3)
    dW, db, dX = oracle.gcn_backward(rp, c, val, X, W, G)
    loss = lambda X_, W_, b_: float(np.sum(oracle.gcn_forward(rp, c, val, X_, W_, b_) * G))
    args = [X, W, b]
    rng = np.random.default_rng(1)
    for idx, ref_arr in enumerate((dX, dW, db)):
        for _ in range(6):
            pos = tuple(rng.integers(0, s) for s in args[idx].shape)
            hi, lo = args[idx].copy(), args[idx].copy()
            hi[pos] += 1e-6
            lo[pos] -= 1e-6
            fd = (loss(*[hi if t == idx else a for t, a in enumerate(args)])
                  - loss(*[lo if t == idx else a for t, a in enumerate(args)])) / 2e-6
            assert abs(fd - ref_arr[pos]) <= 1e-6 * (1 + abs(ref_arr[pos]))


def test_edge_softmax_rows_sum_to_one_and_grad_rows_sum_to_zero():
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=2)
    fw = oracle.gat_forward(rp, c, X, W, a_src, a_dst, b, h, 0.2)
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    sums = np.zeros((rp.size - 1, h))
    np.add.at(sums, rows, fw["alpha"])
    np.testing.assert_allclose(sums, 1.0, rtol=1e-14)
    assert fw["alpha"].min() > 0
    # slope 1 makes LeakyReLU the identity, so ds_i = sum_e g_w = 0 for every row
    bw = oracle.gat_backward(rp, c, X, W, a_src, a_dst, G, h, 1.0)
    assert np.abs(bw["ds"]).max() < 1e-13
    # total gradient mass reaching d equals that reaching s (both sum g_y over all entries)
    bw = oracle.gat_backward(rp, c, X, W, a_src, a_dst, G, h, 0.2)
    np.testing.assert_allclose(bw["dd"].sum(axis=0), bw["ds"].sum(axis=0), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["gy"].sum(axis=0), bw["ds"].sum(axis=0), rtol=1e-10, atol=1e-12)


def test_gat_zero_attention_is_mean_aggregation():
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=3)
    z = np.zeros_like(a_src)
    fw = oracle.gat_forward(rp, c, X, W, z, z, None, h, 0.2)
    A = dense_pattern(rp, c)
    np.testing.assert_allclose(fw["Y"], (A / A.sum(axis=1, keepdims=True)) @ X @ W, rtol=1e-12, atol=1e-13)


def test_leaky_relu_derivative_at_a_logit_of_exactly_zero_is_the_slope():
    """Sec. "GAT Backward Pass": the LeakyReLU derivative is beta for y <= 0, so at y = 0 it is beta, not 1.
    With a_src = a_dst = 0 every logit is exactly 0 in double and in float: alpha = 1/deg, no mask bit is set,
    and beta multiplies every edge gradient.  Closed form, written here with dense matrices:
      g_alpha = (G_p M_p^T) on the pattern, g_w = (g_alpha - rowmean) / deg, g_y = beta g_w,
      ds = 0, dd_j = column sums of g_y, da_src = 0, da_dst_p = sum_j dd_j m_j.
    A derivative of 1 at zero (the mistake `y >= 0`) would scale da_dst by 1 / beta.  Both sign-decision
    branches of the oracle (double, and float s + d) are held to it, and torch's autograd of
    leaky_relu at 0 (a library routine with the same convention) gives the same numbers."""
    beta = 0.2
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=21)
    n = X.shape[0]
    zero = np.zeros_like(a_src)
    A = dense_pattern(rp, c)
    deg = A.sum(axis=1)
    M = (X @ W).reshape(n, h, k)
    G3 = G.reshape(n, h, k)
    da_dst = np.zeros((h, k))
    dd = np.zeros((n, h))
    for p in range(h):
        ga = (G3[:, p, :] @ M[:, p, :].T) * A                    # g_alpha on the pattern
        gw = (ga - (ga.sum(axis=1) / deg)[:, None]) * A / deg[:, None]
        gy = beta * gw
        assert abs(gy.sum(axis=1)).max() < 1e-12                 # ds = 0
        dd[:, p] = gy.sum(axis=0)
        da_dst[p] = dd[:, p] @ M[:, p, :]
    assert np.abs(da_dst).max() > 1e-2                           # the pin is not vacuous
    fw = oracle.gat_forward(rp, c, X, W, zero, zero, None, h, beta)
    assert not fw["mask"].any() and np.all(fw["s"] == 0) and np.all(fw["d"] == 0)
    bw = oracle.gat_backward(rp, c, X, W, zero, zero, G, h, beta)                       # decision in double
    z32 = np.zeros((n, h), np.float32)
    bw32 = oracle.gat_backward_cached(rp, c, X, W, zero, zero, G, M.astype(np.float32), z32, z32, beta)
    for name, got in (("double", bw), ("float", bw32)):
        tol = dict(rtol=1e-12, atol=1e-13) if name == "double" else dict(rtol=1e-5, atol=1e-6)   # M rounded to float
        np.testing.assert_allclose(got["da_dst"], da_dst, err_msg=name, **tol)
        np.testing.assert_allclose(got["dd"], dd, err_msg=name, **tol)
        np.testing.assert_allclose(got["da_src"], 0.0, atol=1e-12 if name == "double" else 1e-6, err_msg=name)
        np.testing.assert_allclose(got["ds"], 0.0, atol=1e-12 if name == "double" else 1e-6, err_msg=name)
    tens = [torch.tensor(a, requires_grad=True) for a in (X, W, zero, zero, b)]
    (_torch_dense_gat(rp, c, *tens, h, k, beta) * torch.tensor(G)).sum().backward()
    np.testing.assert_allclose(tens[3].grad.numpy(), da_dst, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw["dW"], tens[1].grad.numpy(), rtol=1e-10, atol=1e-11)


def test_gat_identical_heads_give_identical_blocks_and_head_order():
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=6, h=3, k=4)
    W1 = np.tile(W[:, :k], (1, h))
    a1, a2 = np.tile(a_src[:1], (h, 1)), np.tile(a_dst[:1], (h, 1))
    Y = oracle.gat_forward(rp, c, X, W1, a1, a2, None, h, 0.2)["Y"]
    for p in range(1, h):
        np.testing.assert_allclose(Y[:, p * k:(p + 1) * k], Y[:, :k], rtol=1e-14)
    # a multi-head layer is the concatenation of single-head layers (Sec. GAT Forward Pass)
    Yall = oracle.gat_forward(rp, c, X, W, a_src, a_dst, b, h, 0.2)["Y"]
    for p in range(h):
        Yp = oracle.gat_forward(rp, c, X, W[:, p * k:(p + 1) * k], a_src[p:p + 1], a_dst[p:p + 1],
                                b[p * k:(p + 1) * k], 1, 0.2)["Y"]
        np.testing.assert_allclose(Yall[:, p * k:(p + 1) * k], Yp, rtol=1e-13, atol=1e-14)


def test_gat_single_node_and_src_dst_roles():
    rp, c, _ = oracle.add_self_loops_degree(np.zeros(2, np.int32), np.zeros(0, np.int32))
    X, W = np.array([[1.0, -2.0]]), np.array([[0.5, 1.0], [3.0, -1.0]])
    a = np.array([[0.3, -0.7]])
    fw = oracle.gat_forward(rp, c, X, W, a, a, np.array([0.25, 0.5]), 1, 0.2)
    np.testing.assert_allclose(fw["Y"], X @ W + [0.25, 0.5])
    # a_src must pair with the row node: on a 2-node graph where row 0 holds {0, 1} and row 1 holds {1},
    # row 0's two logits differ only through d (the column node's term)
    rp2, c2 = np.array([0, 2, 3], np.int32), np.array([0, 1, 1], np.int32)
    X2 = np.array([[1.0, 0.0], [0.0, 1.0]])
    fw = oracle.gat_forward(rp2, c2, X2, np.eye(2), np.array([[5.0, 0.0]]), np.array([[0.0, 2.0]]), None, 1, 0.2)
    # s = [5, 0], d = [0, 2]; row 0 logits: 5+0, 5+2 -> softmax of (5, 7)
    e = np.exp([5.0 - 7.0, 0.0])
    np.testing.assert_allclose(fw["alpha"][:2, 0], e / e.sum(), rtol=1e-14)
    np.testing.assert_allclose(fw["alpha"][2, 0], 1.0)


def test_gat_cached_backward_equals_recompute_when_inputs_are_float32_exact():
    slope = 0.2
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=12)
    fw = oracle.gat_forward(rp, c, X, W, a_src, a_dst, None, h, slope)
    M32, s32, d32 = (fw[t].astype(np.float32) for t in ("M", "s", "d"))
    got = oracle.gat_backward_cached(rp, c, X, W, a_src, a_dst, G, M32, s32, d32, slope)
    ref = oracle.gat_backward(rp, c, X, W, a_src, a_dst, G, h, slope)
    for name in ("dX", "dW", "da_src", "da_dst"):
        np.testing.assert_allclose(got[name], ref[name], rtol=2e-5, atol=2e-5, err_msg=name)


def test_tie_band_switches_only_near_zero_logits():
    rp, c, X, W, a_src, a_dst, b, G, h, k = _gat_case(seed=14)
    fw0 = oracle.gat_forward(rp, c, X, W, a_src, a_dst, None, h, 0.2)
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    y = fw0["s"][rows] + fw0["d"][c]
    eps = np.sort(np.abs(y).ravel())[5] * 1.0001                 # six logits fall inside the band
    lo = oracle.gat_forward(rp, c, X, W, a_src, a_dst, None, h, 0.2, tie_eps=eps, tie_mode=-1)
    hi = oracle.gat_forward(rp, c, X, W, a_src, a_dst, None, h, 0.2, tie_eps=eps, tie_mode=+1)
    inside = np.abs(y) <= eps
    assert inside.sum() == 6
    assert np.all(lo["mask"][inside] == 0) and np.all(hi["mask"][inside] == 1)
    np.testing.assert_array_equal(lo["mask"][~inside], fw0["mask"][~inside])
    np.testing.assert_array_equal(hi["mask"][~inside], (y > 0)[~inside])


# ------------------------------------------------------------------ loss
def test_elu_and_its_gradient_against_torch():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((40, 7)) * 2.0
    x[0, :3] = [0.0, -1e-9, 1e-9]
    g = rng.standard_normal(x.shape)
    t = torch.tensor(x, requires_grad=True)
    y = torch.nn.functional.elu(t)
    (y * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(oracle.elu(x), y.detach().numpy(), rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(oracle.elu_grad_from_output(g, oracle.elu(x)), t.grad.numpy(), rtol=1e-13, atol=1e-15)
    assert oracle.elu(np.array([-50.0]))[0] == pytest.approx(-1.0, abs=1e-15)      # saturates, no overflow
    assert oracle.elu(np.array([700.0]))[0] == 700.0


def test_two_layer_gat_with_elu_and_squared_error_against_torch_autograd():
    """The paper's GAT network (Sec. 4): GAT -> ELU -> GAT, squared error; every gradient of the
    chained oracle calls against autograd on the dense masked-softmax form."""
    slope, h, k1, k2 = 0.2, 2, 3, 2
    rng = np.random.default_rng(11)
    rowptr, col = small_graph(n=23, q=90, seed=211, diagonal=False)
    rp, c, _ = oracle.add_self_loops_degree(rowptr, col)
    n, m = 23, 4
    X = rng.standard_normal((n, m))
    W1, W2 = rng.standard_normal((m, h * k1)) * 0.7, rng.standard_normal((h * k1, h * k2)) * 0.7
    a1s, a1d, a2s, a2d = (rng.standard_normal((h, kk)) for kk in (k1, k1, k2, k2))
    b1, b2 = rng.standard_normal(h * k1), rng.standard_normal(h * k2)
    T = rng.standard_normal((n, h * k2))
    params = (X, W1, a1s, a1d, b1, W2, a2s, a2d, b2)
    tens = [torch.tensor(a, requires_grad=True) for a in params]
    tX, tW1, ta1s, ta1d, tb1, tW2, ta2s, ta2d, tb2 = tens
    H = torch.nn.functional.elu(_torch_dense_gat(rp, c, tX, tW1, ta1s, ta1d, tb1, h, k1, slope))
    Z = _torch_dense_gat(rp, c, H, tW2, ta2s, ta2d, tb2, h, k2, slope)
    loss_t = 0.5 * ((Z - torch.tensor(T)) ** 2).sum()
    loss_t.backward()

    f1 = oracle.gat_forward(rp, c, X, W1, a1s, a1d, b1, h, slope)
    H1 = oracle.elu(f1["Y"])
    f2 = oracle.gat_forward(rp, c, H1, W2, a2s, a2d, b2, h, slope)
    loss, dZ = oracle.sum_squared_error(f2["Y"], T)
    g2 = oracle.gat_backward(rp, c, H1, W2, a2s, a2d, dZ, h, slope)
    dpre = oracle.elu_grad_from_output(g2["dX"], H1)
    g1 = oracle.gat_backward(rp, c, X, W1, a1s, a1d, dpre, h, slope)
    assert loss == pytest.approx(float(loss_t.detach()), rel=1e-12)
    np.testing.assert_allclose(f2["Y"], Z.detach().numpy(), rtol=1e-11, atol=1e-12)
    got = (g1["dX"], g1["dW"], g1["da_src"], g1["da_dst"], g1["db"], g2["dW"], g2["da_src"], g2["da_dst"], g2["db"])
    for name, a, t in zip("dX dW1 da1s da1d db1 dW2 da2s da2d db2".split(), got, tens):
        np.testing.assert_allclose(a, t.grad.numpy().reshape(a.shape), rtol=1e-9, atol=1e-10, err_msg=name)


def test_mean_and_gin_weights_against_dense_definitions():
    """Mean aggregation is D^-1 (A + I) X (rows of the weight matrix sum to one, the layer output is the
    neighbourhood mean); the GIN sum is (A + (1 + eps) I) X."""
    rowptr, col = small_graph(n=29, q=120, seed=77, diagonal=False)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    n = rp.size - 1
    pat = dense_pattern(rp, c)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, 5))
    mean = oracle.aggregator_weights(rp, c, deg, "mean")
    got = oracle.spmm(rp, c, mean, X)
    ref = np.stack([X[np.flatnonzero(pat[i])].mean(axis=0) for i in range(n)])
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(np.add.reduceat(mean, rp[:-1]), 1.0, rtol=1e-14)
    eps = 0.25
    gin = oracle.aggregator_weights(rp, c, deg, "gin", eps)
    A_plain = pat - np.eye(n)                                      # the pattern without the added diagonal
    np.testing.assert_allclose(oracle.spmm(rp, c, gin, X), (1 + eps) * X + A_plain @ X, rtol=1e-13, atol=1e-13)


def test_sage_layer_against_node_loop_and_autograd():
    """GraphSAGE with the mean aggregator: each output row is x_i W_self + mean over the neighbourhood of x_j
    times W_neigh (a loop over nodes), and the gradients are those of torch autograd on the dense form."""
    rowptr, col = small_graph(n=23, q=90, seed=5, diagonal=False)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    n = rp.size - 1
    val = oracle.aggregator_weights(rp, c, deg, "mean")
    rng = np.random.default_rng(8)
    X, Ws, Wn = rng.standard_normal((n, 6)), rng.standard_normal((6, 4)), rng.standard_normal((6, 4))
    b, G = rng.standard_normal(4), rng.standard_normal((n, 4))
    Y = oracle.sage_forward(rp, c, val, X, Ws, Wn, b, relu=True)
    for i in range(n):
        nb = c[rp[i]:rp[i + 1]]
        row = X[i] @ Ws + X[nb].mean(axis=0) @ Wn + b
        np.testing.assert_allclose(Y[i], np.maximum(row, 0.0), rtol=1e-13, atol=1e-14)
    A = dense_pattern(rp, c)
    A = torch.tensor(A / A.sum(axis=1, keepdims=True))
    Xt, Wst, Wnt, bt = (torch.tensor(a, requires_grad=True) for a in (X, Ws, Wn, b))
    Yt = torch.relu(Xt @ Wst + A @ Xt @ Wnt + bt)
    Yt.backward(torch.tensor(G))
    dWs, dWn, db, dX = oracle.sage_backward(rp, c, val, X, Ws, Wn, G, Y_relu=Y)
    for got, ref in ((dWs, Wst.grad), (dWn, Wnt.grad), (db, bt.grad), (dX, Xt.grad)):
        np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-13)
    # without the neighbour weight the layer is a dense layer; without the self weight a GCN-shaped one
    np.testing.assert_allclose(oracle.sage_forward(rp, c, val, X, Ws, np.zeros_like(Wn)), X @ Ws, rtol=1e-14)
    np.testing.assert_allclose(oracle.sage_forward(rp, c, val, X, np.zeros_like(Ws), Wn),
                               oracle.gcn_forward(rp, c, val, X, Wn), rtol=1e-12, atol=1e-13)


def test_other_storage_formats_against_the_dense_product():
    """App. D: the same matrix in coordinate, ELLPACK and hybrid form gives the same product as its dense
    form; the hybrid's two parts hold every entry exactly once; an ELLPACK as wide as the longest row has
    no coordinate part; unsorted coordinate triples and duplicates are fine."""
    rowptr, col = small_graph(n=31, q=140, seed=12, diagonal=False)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    n = rp.size - 1
    rng = np.random.default_rng(2)
    val = rng.standard_normal(c.size)
    Bm = rng.standard_normal((n, 7))
    A = np.zeros((n, n))
    rows = np.repeat(np.arange(n), np.diff(rp))
    A[rows, c] = val
    ref = A @ Bm
    np.testing.assert_allclose(oracle.spmm_coo(n, rows, c, val, Bm), ref, rtol=1e-13, atol=1e-13)
    perm = rng.permutation(c.size)
    np.testing.assert_allclose(oracle.spmm_coo(n, rows[perm], c[perm], val[perm], Bm), ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm_coo(n, np.r_[rows, rows], np.r_[c, c], np.r_[val, val], Bm), 2 * ref,
                               rtol=1e-13, atol=1e-13)
    longest = int(np.diff(rp).max())
    for t in (0, 1, 3, longest, longest + 2):
        ec, ev, rr, rc, rv = oracle.csr_to_hybrid(rp, c, val, t)
        assert ec.shape == (t, n)
        assert (ec >= 0).sum() + rr.size == c.size
        assert (rr.size == 0) == (t >= longest)
        assert np.all(ev[ec < 0] == 0)
        got = oracle.spmm_ell(ec, ev, Bm) + oracle.spmm_coo(n, rr, rc, rv, Bm)
        np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
        # a row's stored slots come first, in CSR order
        for i in (0, n // 2, n - 1):
            k = min(t, rp[i + 1] - rp[i])
            assert np.array_equal(ec[:k, i], c[rp[i]:rp[i] + k]) and np.all(ec[k:, i] == -1)


def test_ellpack_is_mostly_padding_on_the_papers_graphs():
    """App. E.1: with the maximum degrees 168 (Cora) and 436 (Arxiv) the ELLPACK value matrices consist of
    more than 96 % zeros."""
    assert oracle.ell_padding_fraction(2708, 10556, 168) > 0.96
    assert oracle.ell_padding_fraction(169343, 1166243, 436) > 0.96
    assert abs(oracle.ell_padding_fraction(10, 40, 4)) < 1e-15


def test_softmax_xent_against_torch():
    rng = np.random.default_rng(4)
    Z = rng.standard_normal((50, 7)) * 3
    lab = rng.integers(0, 7, size=50).astype(np.int32)
    Zt = torch.tensor(Z, requires_grad=True)
    L = torch.nn.functional.cross_entropy(Zt, torch.tensor(lab, dtype=torch.long), reduction="sum")
    L.backward()
    loss, dZ = oracle.softmax_xent(Z, lab)
    assert abs(loss - L.item()) < 1e-10
    np.testing.assert_allclose(dZ, Zt.grad.numpy(), rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ the paper's printed numbers
def test_spmm_operational_intensity_table():
    """App. E.1, table of SpMM operational intensities (dense width 64)."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "spmm_op_intensity.txt")) if not ln.startswith("#")]
    graphs = {"cora": (2708, 10556, 168), "arxiv": (169343, 1166243, 436)}
    assert len(rows) == 8
    for fmt, graph, printed in rows:
        n, q, p = graphs[graph]
        got = oracle.spmm_operational_intensity(fmt, n, q, 64, p)
        assert abs(got - float(printed)) < 5e-4, (fmt, graph, got, printed)
