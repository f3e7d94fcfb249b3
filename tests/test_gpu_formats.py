"""Coordinate, ELLPACK and hybrid storage (App. D) through the C ABI: conversions bit-exact against the
oracle, SpMM within the fp32 tolerance."""
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


def graph(scale, seed, directed=False):
    s = synth.streams(seed)
    rowptr, col = synth.rmat_graph(scale, 8, directed, s["graph"], s["relabel"])
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = synth.normal(s["X"], c.size)
    return rp, c, val, s


def to_hybrid(B, rp, c, val, t):
    """CSR -> hybrid on the device; returns device arrays and the two counts."""
    n = rp.size - 1
    rp_d, c_d = dev(rp), dev(c)
    val_d = None if val is None else dev(val)
    rest_ptr = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    ws = B.alloc(B.gnn_hyb_workspace_bytes(n))
    rest, longest = B.gnn_csr_hyb_count(n, rp_d, t, rest_ptr, ws)
    ell_col = torch.full((max(t, 1), n), 7, dtype=torch.int32, device="cuda")
    ell_val = torch.full((max(t, 1), n), float("nan"), dtype=torch.float32, device="cuda")
    coo = [torch.full((max(rest, 1),), -5, dtype=torch.int32, device="cuda") for _ in range(2)]
    coo_val = torch.full((max(rest, 1),), float("nan"), dtype=torch.float32, device="cuda")
    B.gnn_csr_to_hyb(n, t, rp_d, c_d, val_d, rest_ptr, ell_col, ell_val, coo[0], coo[1], coo_val)
    torch.cuda.synchronize()
    return dict(n=n, t=t, rest=rest, longest=longest, rest_ptr=rest_ptr, ell_col=ell_col, ell_val=ell_val,
                coo_row=coo[0], coo_col=coo[1], coo_val=coo_val)


@pytest.mark.parametrize("t", [0, 1, 5, 16, 40])
def test_conversion_is_bit_exact(B, t):
    rp, c, val, _ = graph(9, 71)
    h = to_hybrid(B, rp, c, val, t)
    ec, ev, rr, rc, rv = oracle.csr_to_hybrid(rp, c, val, t)
    lens = np.diff(rp)
    assert h["longest"] == lens.max()
    assert h["rest"] == rr.size == np.maximum(lens - t, 0).sum()
    assert np.array_equal(host(h["rest_ptr"]), np.r_[0, np.cumsum(np.maximum(lens - t, 0))])
    if t:
        assert np.array_equal(host(h["ell_col"]), ec)
        assert np.array_equal(host(h["ell_val"]), ev.astype(np.float32))
    assert np.array_equal(host(h["coo_row"])[:rr.size], rr)
    assert np.array_equal(host(h["coo_col"])[:rr.size], rc)
    assert np.array_equal(host(h["coo_val"])[:rr.size], rv.astype(np.float32))


def test_pattern_without_values_gets_ones(B):
    rp, c, _, _ = graph(8, 72)
    h = to_hybrid(B, rp, c, None, 4)
    ec, ev, rr, rc, rv = oracle.csr_to_hybrid(rp, c, None, 4)
    assert np.array_equal(host(h["ell_val"]), ev.astype(np.float32))
    assert np.all(host(h["coo_val"])[:rr.size] == 1.0)


@pytest.mark.parametrize("f", [1, 6, 16, 47, 64, 128, 300, 512])
def test_spmm_in_every_format(B, f):
    rp, c, val, s = graph(10, 73, directed=True)
    n = rp.size - 1
    Bm = synth.normal(s["dY"], n, f)
    ref = oracle.spmm(rp, c, val, Bm)
    rows = np.repeat(np.arange(n, dtype=np.int32), np.diff(rp))
    Bd = dev(Bm)
    # coordinate, sorted and shuffled, and accumulating onto what C holds
    for order in (np.arange(c.size), np.random.default_rng(f).permutation(c.size)):
        C = torch.full((n, f), float("nan"), dtype=torch.float32, device="cuda")
        B.gnn_spmm_coo(n, c.size, dev(rows[order]), dev(c[order]), dev(val[order]), Bd, f, C)
        assert_close(host(C), ref, f"coo f={f}")
    C0 = synth.normal(s["W"], n, f)
    C = dev(C0)
    B.gnn_spmm_coo(n, c.size, dev(rows), dev(c), dev(val), Bd, f, C, accumulate=True)
    assert_close(host(C), ref + C0, f"coo accumulate f={f}")
    # ELLPACK as wide as the longest row, and hybrids
    longest = int(np.diff(rp).max())
    for t in (longest, 0, 3, 16, 33):
        h = to_hybrid(B, rp, c, val, t)
        C = torch.full((n, f), float("nan"), dtype=torch.float32, device="cuda")
        if t == longest:
            assert h["rest"] == 0
            B.gnn_spmm_ell(n, t, h["ell_col"], h["ell_val"], Bd, f, C)
        else:
            B.gnn_spmm_hyb(n, t, h["ell_col"], h["ell_val"], h["rest"], h["coo_row"], h["coo_col"], h["coo_val"],
                           Bd, f, C)
        assert_close(host(C), ref, f"ell/hyb t={t} f={f}")


def test_ell_is_deterministic_and_handles_ragged_row_tiles(B):
    """n is not a multiple of the kernel's 64-row tile; two runs agree bit for bit."""
    rng = np.random.default_rng(5)
    n, t, f = 1000 + 37, 9, 40
    lens = rng.integers(0, t + 1, n)
    rp = np.r_[0, np.cumsum(lens)].astype(np.int32)
    c = rng.integers(0, n, rp[-1]).astype(np.int32)
    val = rng.standard_normal(rp[-1]).astype(np.float32)
    Bm = rng.standard_normal((n, f), dtype=np.float32)
    h = to_hybrid(B, rp, c, val, t)
    assert h["rest"] == 0 and h["longest"] == lens.max()
    outs = []
    for _ in range(2):
        C = torch.full((n, f), float("nan"), dtype=torch.float32, device="cuda")
        B.gnn_spmm_ell(n, t, h["ell_col"], h["ell_val"], dev(Bm), f, C)
        outs.append(host(C))
    assert np.array_equal(outs[0], outs[1])
    assert_close(outs[0], oracle.spmm(rp, c, val, Bm), "ell")


def test_graph_without_entries(B):
    n, f = 5, 8
    rp = np.zeros(n + 1, np.int32)
    h = to_hybrid(B, rp, np.zeros(0, np.int32), None, 2)
    assert h["rest"] == 0 and h["longest"] == 0
    assert np.all(host(h["ell_col"]) == -1)
    C = torch.full((n, f), float("nan"), dtype=torch.float32, device="cuda")
    Bd = torch.ones((n, f), dtype=torch.float32, device="cuda")
    B.gnn_spmm_hyb(n, 2, h["ell_col"], h["ell_val"], 0, None, None, None, Bd, f, C)
    assert np.all(host(C) == 0)
    B.gnn_spmm_coo(n, 0, None, None, None, Bd, f, C)
    assert np.all(host(C) == 0)
