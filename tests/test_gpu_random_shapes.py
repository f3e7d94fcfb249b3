"""Seeded sweep over odd shapes: node counts, densities and feature widths that are not multiples of any
tile, vector or wavefront size, through the layer entry points and the operators, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_12093_amd import synth
from tests._util import assert_close, dev, host
from tests.test_gpu_gcn import run_layer, oracle_layer, schemes
from tests.test_gpu_gat import Layer, oracle_graph, ambiguous_logits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2308_12093_amd import binding
    return binding


@pytest.fixture(scope="module")
def G():
    from paper_2308_12093_amd import graphs
    return graphs


def random_graph(rng, n, q, directed):
    rowptr, col = synth.random_directed_graph(n, q, rng)
    if directed:
        return rowptr, col
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    r, c = np.concatenate([rows, col]), np.concatenate([col, rows])
    key = np.unique(r.astype(np.int64) * n + c)
    return synth.coo_to_csr(n, (key // n).astype(np.int64), (key % n).astype(np.int64))


GCN_CASES = [(seed, n, q, m, k) for seed, (n, q, m, k) in enumerate([
    (1, 0, 1, 1), (2, 1, 3, 2), (63, 100, 5, 7), (65, 300, 33, 31), (129, 64, 17, 130), (257, 2000, 130, 17),
    (500, 499, 64, 1), (777, 9000, 1, 64), (1023, 5000, 47, 100), (1500, 20000, 96, 260), (4097, 30000, 12, 12),
    (3000, 100, 36, 68)])]


@pytest.mark.parametrize("seed,n,q,m,k", GCN_CASES)
def test_gcn_layer_odd_shapes(B, G, seed, n, q, m, k):
    rng = np.random.default_rng(1000 + seed)
    directed = seed % 2 == 1
    rowptr, col = random_graph(rng, n, min(q, n * (n - 1)), directed)
    X = rng.standard_normal((n, m), dtype=np.float32)
    W = rng.standard_normal((m, k), dtype=np.float32) / np.float32(np.sqrt(m))
    b = rng.standard_normal(k, dtype=np.float32)
    dY = rng.standard_normal((n, k), dtype=np.float32)
    g = G.gcn_graph(rowptr, col, symmetric=not directed)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, c, deg)
    rY, rW, rb, rX = oracle_layer(rp, c, val, X, W, b, dY, True, False)
    for name in ("tf_fp", "pf_sp_cache", "pf_sp_nocache"):
        Y, gW, gb, gX, _ = run_layer(B, g, X, W, b, dY, True, False, schemes(B)[name])
        assert_close(Y, rY, f"{name} Y")
        assert_close(gW, rW, f"{name} dW")
        assert_close(gb, rb, f"{name} db")
        assert_close(gX, rX, f"{name} dX")


GAT_CASES = [(seed, n, q, m, h, k) for seed, (n, q, m, h, k) in enumerate([
    (1, 0, 3, 1, 1), (2, 2, 2, 2, 3), (67, 200, 9, 3, 7), (130, 900, 20, 5, 4), (300, 2500, 33, 2, 33),
    (513, 4000, 16, 8, 16), (1000, 7000, 40, 1, 64), (2049, 12000, 7, 7, 9)])]


@pytest.mark.parametrize("seed,n,q,m,h,k", GAT_CASES)
def test_gat_layer_odd_shapes(B, G, seed, n, q, m, h, k):
    rng = np.random.default_rng(2000 + seed)
    rowptr, col = random_graph(rng, n, min(q, n * (n - 1)), True)
    f = h * k
    t = dict(X=rng.standard_normal((n, m), dtype=np.float32),
             W=(rng.standard_normal((m, f), dtype=np.float32) / np.float32(np.sqrt(m))),
             a_src=rng.standard_normal((h, k), dtype=np.float32) * np.float32(0.5),
             a_dst=rng.standard_normal((h, k), dtype=np.float32) * np.float32(0.5),
             b=rng.standard_normal(f, dtype=np.float32), dY=rng.standard_normal((n, f), dtype=np.float32))
    rp, c = oracle_graph(rowptr, col)
    fw = oracle.gat_forward(rp, c, t["X"], t["W"], t["a_src"], t["a_dst"], t["b"], h, 0.2)
    if ambiguous_logits(fw, rp, c, 1e-5):
        pytest.skip("a logit of this seeded case is too close to zero for float and double to agree on its sign")
    bw = oracle.gat_backward(rp, c, t["X"], t["W"], t["a_src"], t["a_dst"], t["dY"], h, 0.2)
    for variant in (B.GNN_CACHE_NONE, B.GNN_CACHE_GAT_FEAT_EDGE):
        layer = Layer(B, G, rowptr, col, t, h, variant)
        assert_close(layer.forward(), fw["Y"], "Y")
        got = layer.backward()
        for name in ("dW", "da_src", "da_dst", "dX"):
            assert_close(got[name], bw[name].reshape(got[name].shape), f"variant {variant} {name}")
