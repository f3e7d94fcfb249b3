"""Parity of the single operators (preprocessing, SpMM, GEMM) with the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_12093_amd import synth
from tests._util import assert_close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2308_12093_amd import binding
    return binding


@pytest.fixture(scope="module")
def G():
    from paper_2308_12093_amd import graphs
    return graphs


def rmat_small(scale=12, deg=14, directed=False, seed=1):
    s = synth.streams(seed)
    return synth.rmat_graph(scale, deg, directed, s["graph"], s["relabel"])


# ---------------------------------------------------------------- preprocessing (bit-exact)
@pytest.mark.parametrize("case", ["rmat", "with_diagonal", "empty", "one_node"])
def test_self_loops_degree_normalize(B, G, case):
    if case == "rmat":
        rowptr, col = rmat_small()
    elif case == "with_diagonal":
        rowptr, col = synth.random_directed_graph(700, 6000, np.random.default_rng(5), allow_diagonal=True)
    elif case == "empty":
        rowptr, col = np.zeros(1001, np.int32), np.zeros(0, np.int32)
    else:
        rowptr, col = np.zeros(2, np.int32), np.zeros(0, np.int32)
    n = rowptr.size - 1
    rp_o, c_o, deg_o = oracle.add_self_loops_degree(rowptr, col)
    rp, c, deg = G.add_self_loops(n, dev(rowptr), dev(col))
    np.testing.assert_array_equal(host(rp), rp_o)
    np.testing.assert_array_equal(host(c), c_o)
    np.testing.assert_array_equal(host(deg), deg_o)
    val = torch.empty(c.numel(), dtype=torch.float32, device="cuda")
    B.gnn_gcn_normalize(n, rp, c, deg, val)
    assert_close(host(val), oracle.gcn_normalize(rp_o, c_o, deg_o), "val", tol=1e-6)


@pytest.mark.parametrize("case", ["rmat_directed", "rmat_big", "tiny", "empty"])
def test_csr_transpose_bit_exact(B, G, case):
    if case == "rmat_directed":
        rowptr, col = rmat_small(12, 14, directed=True)
    elif case == "rmat_big":
        rowptr, col = rmat_small(17, 6, directed=True, seed=3)      # three radix passes, many tiles, ragged tail
    elif case == "tiny":
        rowptr, col = synth.random_directed_graph(5, 11, np.random.default_rng(0), allow_diagonal=True)
    else:
        rowptr, col = np.zeros(8, np.int32), np.zeros(0, np.int32)
    n = rowptr.size - 1
    colptr_o, row_o, perm_o = oracle.csr_transpose(rowptr, col)
    colptr, row, perm = G.transpose(n, dev(rowptr), dev(col))
    np.testing.assert_array_equal(host(colptr), colptr_o)
    np.testing.assert_array_equal(host(row), row_o)
    np.testing.assert_array_equal(host(perm), perm_o)
    # twice the same bits
    colptr2, row2, perm2 = G.transpose(n, dev(rowptr), dev(col))
    assert torch.equal(perm, perm2) and torch.equal(row, row2)
    np.testing.assert_array_equal(host(G.expand(n, dev(rowptr), col.size)), np.repeat(np.arange(n), np.diff(rowptr)))


# ---------------------------------------------------------------- SpMM
def run_spmm(B, rowptr, col, val, Bm, bias=None, relu=False, balanced=True):
    n = rowptr.size - 1
    f = Bm.shape[1]
    d_rp, d_c = dev(rowptr), dev(col)
    d_val = None if val is None else dev(val.astype(np.float32))
    erow = None
    if balanced:
        erow = torch.empty(max(col.size, 1), dtype=torch.int32, device="cuda")
        B.gnn_expand_ptr(n, col.size, d_rp, erow)
    ws = B.alloc(B.gnn_spmm_workspace_bytes(n, col.size, f))
    C = torch.full((n, f), float("nan"), dtype=torch.float32, device="cuda")
    B.gnn_spmm_csr(n, col.size, d_rp, d_c, d_val, erow, dev(Bm), f, C,
                   None if bias is None else dev(bias), relu, ws)
    torch.cuda.synchronize()
    return host(C)


@pytest.mark.parametrize("f", [4, 16, 47, 64, 100, 128, 256, 512, 1024, 1030, 3])
@pytest.mark.parametrize("balanced", [True, False])
def test_spmm_matches_oracle(B, f, balanced):
    rowptr, col = rmat_small()                     # hubs: rows far longer than a segment
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, c, deg).astype(np.float32)
    rng = np.random.default_rng(f)
    Bm = rng.standard_normal((rp.size - 1, f), dtype=np.float32)
    ref = oracle.spmm(rp, c, val, Bm)
    assert_close(run_spmm(B, rp, c, val, Bm, balanced=balanced), ref, f"spmm f={f}")


@pytest.mark.parametrize("f", [4, 5, 7, 30, 47, 130, 301])
def test_spmm_rows_that_are_not_16_byte_aligned(B, f):
    """Ragged widths, and operands that start 4 bytes into an allocation: the four-wide kernel moves whole
    rows with unaligned 16-byte accesses and the ragged end of a row value by value; bias and ReLU included."""
    rowptr, col = rmat_small()
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    n = rp.size - 1
    val = oracle.gcn_normalize(rp, c, deg).astype(np.float32)
    rng = np.random.default_rng(100 + f)
    Bm = rng.standard_normal((n, f), dtype=np.float32)
    bias = rng.standard_normal(f, dtype=np.float32)
    ref = np.maximum(oracle.spmm(rp, c, val, Bm) + bias, 0.0)
    d_rp, d_c, d_val = dev(rp), dev(c), dev(val)
    erow = torch.empty(c.size, dtype=torch.int32, device="cuda")
    B.gnn_expand_ptr(n, c.size, d_rp, erow)
    ws = B.alloc(B.gnn_spmm_workspace_bytes(n, c.size, f))
    for shift_b, shift_c in ((0, 0), (1, 0), (0, 1), (1, 3)):
        Bbuf = torch.zeros(n * f + 4, dtype=torch.float32, device="cuda")
        Cbuf = torch.full((n * f + 4,), float("nan"), dtype=torch.float32, device="cuda")
        Bv, Cv = Bbuf[shift_b:shift_b + n * f].view(n, f), Cbuf[shift_c:shift_c + n * f].view(n, f)
        Bv.copy_(dev(Bm))
        B.gnn_spmm_csr(n, c.size, d_rp, d_c, d_val, erow, Bv, f, Cv, dev(bias), True, ws)
        torch.cuda.synchronize()
        assert_close(host(Cv), ref, f"f={f} shifts {shift_b},{shift_c}")
        out = host(Cbuf)
        assert np.all(np.isnan(out[:shift_c])) and np.all(np.isnan(out[shift_c + n * f:]))   # nothing written outside


def test_spmm_epilogue_unit_weights_and_empty_rows(B):
    rowptr, col = rmat_small(11, 6, directed=True)                 # no self-loops: many empty rows
    assert (np.diff(rowptr) == 0).sum() > 100
    rng = np.random.default_rng(0)
    Bm = rng.standard_normal((rowptr.size - 1, 64), dtype=np.float32)
    bias = rng.standard_normal(64, dtype=np.float32)
    ref = np.maximum(oracle.spmm(rowptr, col, None, Bm) + bias, 0.0)
    for balanced in (True, False):
        assert_close(run_spmm(B, rowptr, col, None, Bm, bias, True, balanced), ref, f"epilogue balanced={balanced}")


def test_spmm_star_graph_row_spans_many_segments(B):
    n = 70001                                                      # row 0 holds every column; the rest only (i, 0)
    rowptr = np.concatenate([[0], n + np.arange(n)]).astype(np.int32)
    col = np.concatenate([np.arange(n), np.zeros(n - 1)]).astype(np.int32)
    rng = np.random.default_rng(1)
    val = rng.standard_normal(col.size).astype(np.float32) / 16
    Bm = rng.standard_normal((n, 16), dtype=np.float32)
    assert_close(run_spmm(B, rowptr, col, val, Bm), oracle.spmm(rowptr, col, val, Bm), "star")


def test_spmm_degenerate_sizes(B):
    rng = np.random.default_rng(2)
    # no entries at all
    out = run_spmm(B, np.zeros(6, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                   rng.standard_normal((5, 8), dtype=np.float32))
    assert np.all(out == 0)
    # one node, one entry
    out = run_spmm(B, np.array([0, 1], np.int32), np.array([0], np.int32), np.array([2.0], np.float32),
                   np.array([[1.5, -1.0, 0.25, 4.0]], np.float32))
    np.testing.assert_allclose(out, [[3.0, -2.0, 0.5, 8.0]])
    # exactly one segment boundary on a row boundary, last segment ragged
    rowptr = np.arange(0, 16 * 41 + 1, 16, dtype=np.int32)
    col = np.tile(np.arange(16, dtype=np.int32), 41)
    Bm = rng.standard_normal((41, 8), dtype=np.float32)
    assert_close(run_spmm(B, rowptr, col, None, Bm), oracle.spmm(rowptr, col, None, Bm), "aligned rows")


def test_spmm_is_deterministic(B):
    rowptr, col = rmat_small()
    rng = np.random.default_rng(3)
    val = rng.standard_normal(col.size).astype(np.float32)
    Bm = rng.standard_normal((rowptr.size - 1, 128), dtype=np.float32)
    a = run_spmm(B, rowptr, col, val, Bm)
    b = run_spmm(B, rowptr, col, val, Bm)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- GEMM
def run_gemm(B, ta, tb, A, Bm, bias=None, relu=False, C0=None):
    M = A.shape[1] if ta else A.shape[0]
    K = A.shape[0] if ta else A.shape[1]
    N = Bm.shape[0] if tb else Bm.shape[1]
    ws = B.alloc(B.gnn_gemm_workspace_bytes(ta, tb, M, N, K))
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda") if C0 is None else dev(C0)
    B.gnn_gemm(ta, tb, M, N, K, dev(A), dev(Bm), C, None if bias is None else dev(bias), relu, ws)
    torch.cuda.synchronize()
    return host(C)


@pytest.mark.parametrize("M,K,N", [(1000, 128, 16), (2048, 512, 16), (777, 100, 47), (1500, 128, 128),
                                   (3000, 128, 512), (129, 33, 65), (1, 1, 1), (4096, 64, 64), (640, 256, 47),
                                   (50, 7, 200)])
def test_gemm_nn_and_nt(B, M, K, N):
    rng = np.random.default_rng(M + K + N)
    A = rng.standard_normal((M, K), dtype=np.float32)
    W = rng.standard_normal((K, N), dtype=np.float32)
    bias = rng.standard_normal(N, dtype=np.float32)
    ref = A.astype(np.float64) @ W.astype(np.float64)
    assert_close(run_gemm(B, 0, 0, A, W), ref, "nn")
    assert_close(run_gemm(B, 0, 0, A, W, bias, True), np.maximum(ref + bias, 0), "nn+bias+relu")
    assert_close(run_gemm(B, 0, 1, A, np.ascontiguousarray(W.T)), ref, "nt")
    # flag word: 4 = add to what C holds (before the ReLU), 1 = ReLU
    C0 = rng.standard_normal((M, N), dtype=np.float32)
    assert_close(run_gemm(B, 0, 0, A, W, None, 4, C0), ref + C0, "nn accumulate")
    assert_close(run_gemm(B, 0, 1, A, np.ascontiguousarray(W.T), bias, 5, C0), np.maximum(ref + bias + C0, 0),
                 "nt accumulate+bias+relu")


@pytest.mark.parametrize("K,M,N", [(50000, 128, 16), (70001, 128, 128), (20000, 100, 256), (9000, 512, 16),
                                   (300000, 64, 64), (100, 5, 3), (4097, 256, 47),
                                   # outputs of 256 x 256 and more take the 128 x 128 tile of the fp64 kernel
                                   (20000, 256, 256), (4097, 300, 260), (9001, 512, 384)])
def test_gemm_tn_split_reduction(B, K, M, N):
    rng = np.random.default_rng(K + M + N)
    A = rng.standard_normal((K, M), dtype=np.float32)
    H = rng.standard_normal((K, N), dtype=np.float32)
    ref = A.astype(np.float64).T @ H.astype(np.float64)
    got = run_gemm(B, 1, 0, A, H)
    assert_close(got, ref, "tn")
    assert np.array_equal(got, run_gemm(B, 1, 0, A, H)), "split-K reduction must be reproducible"


@pytest.mark.parametrize("n,c", [(5000, 47), (1, 1), (3, 2), (257, 16), (1000, 17), (513, 100), (300, 1000),
                                 (70, 3072), (40, 4000), (100000, 47)])
def test_softmax_xent(B, n, c):
    """One lane per row up to 16 classes, lane groups of 2 ... 64 beyond, one thread per row above 3072 classes;
    node counts that end inside a 256-row block and inside a pass."""
    rng = np.random.default_rng(7 + n + c)
    Z = (rng.standard_normal((n, c)) * 3).astype(np.float32)
    lab = rng.integers(0, c, size=n).astype(np.int32)
    dZ = torch.empty((n, c), dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = B.alloc(4 * ((n + 255) // 256))
    B.gnn_softmax_xent(n, c, dev(Z), dev(lab), dZ, loss, ws)
    ref_loss, ref_dZ = oracle.softmax_xent(Z, lab)
    assert_close(host(dZ), ref_dZ, "dZ")
    assert abs(float(loss.item()) - ref_loss) <= 1e-4 * (1 + abs(ref_loss))
