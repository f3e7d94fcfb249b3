"""Parity of sage_layer_fwd / sage_layer_bwd (GraphSAGE, Sec. 3.1 "Generalizability") with the fp64 oracle,
for every order / backward scheme / cache choice, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_12093_amd import synth
from tests._util import assert_close, dev, host
from tests.test_gpu_gcn import schemes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2308_12093_amd import binding
    return binding


@pytest.fixture(scope="module")
def G():
    from paper_2308_12093_amd import graphs
    return graphs


def run_sage(B, g, X, Ws, Wn, b, dY, need_dx, relu, scheme, Ymask=None, constant_input=False, steps=1):
    n, m = X.shape
    k = Ws.shape[1]
    plan = B.Plan(B.GNN_LAYER_SAGE, g.n, g.nnz, m, k, need_input_grad=need_dx, has_bias=b is not None,
                  fuse_relu=relu, constant_input=constant_input, **scheme)
    ws = B.alloc(plan.info.workspace_bytes)
    cache = B.alloc(plan.info.cache_bytes) if plan.info.cache_bytes else None
    Xd, Wsd, Wnd, bd = dev(X), dev(Ws), dev(Wn), None if b is None else dev(b)
    for _ in range(steps):
        Y = torch.full((n, k), float("nan"), dtype=torch.float32, device="cuda")
        B.sage_layer_fwd(plan, g, Xd, Wsd, Wnd, bd, Y, cache, ws)
        torch.cuda.synchronize()
        ws.fill_(0xFF)
        gWs = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda")
        gWn = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda")
        gb = None if b is None else torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
        gX = torch.full((n, m), float("nan"), dtype=torch.float32, device="cuda") if need_dx else None
        mask = None if not relu else (Y if Ymask is None else dev(Ymask))
        B.sage_layer_bwd(plan, g, Xd, Wsd, Wnd, mask, dev(dY), gWs, gWn, gb, gX, cache, ws)
        torch.cuda.synchronize()
        ws.fill_(0xFF)
    return (host(Y), host(gWs), host(gWn), None if gb is None else host(gb), None if gX is None else host(gX),
            plan.info)


def case(seed, scale, m, k, directed):
    s = synth.streams(seed)
    rowptr, col = synth.rmat_graph(scale, 8, directed, s["graph"], s["relabel"])
    n = rowptr.size - 1
    X = synth.normal(s["X"], n, m)
    Ws = synth.glorot_uniform(s["W"], (m, k), m, k)
    Wn = synth.glorot_uniform(s["a_src"], (m, k), m, k)
    return rowptr, col, X, Ws, Wn, synth.normal(s["b"], k), synth.normal(s["dY"], n, k)


@pytest.mark.parametrize("name", ["auto", "tf_fp", "pf_sp_nocache", "pf_sp_cache", "pf_fp", "tf_sp"])
@pytest.mark.parametrize("m,k,directed", [(48, 16, False), (16, 48, True), (100, 47, False), (50, 70, True), (150, 101, False)])
def test_every_scheme_mean_aggregator(B, G, name, m, k, directed):
    rowptr, col, X, Ws, Wn, b, dY = case(61, 10, m, k, directed)
    g = G.gcn_graph(rowptr, col, symmetric=not directed, aggregator=B.GNN_AGG_MEAN)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.aggregator_weights(rp, c, deg, "mean")
    for relu, need_dx in ((False, True), (True, True), (True, False)):
        # both sides take the ReLU sign decisions from the same float32 array: the oracle's forward output
        rY = oracle.sage_forward(rp, c, val, X, Ws, Wn, b, relu)
        Ymask = rY.astype(np.float32) if relu else None
        Y, gWs, gWn, gb, gX, _ = run_sage(B, g, X, Ws, Wn, b, dY, need_dx, relu, schemes(B)[name], Ymask)
        rWs, rWn, rb, rX = oracle.sage_backward(rp, c, val, X, Ws, Wn, dY, Ymask, need_dx)
        tag = f"{name} relu={relu} dx={need_dx}"
        assert_close(Y, rY, tag + " Y")
        assert_close(gWs, rWs, tag + " dW_self")
        assert_close(gWn, rWn, tag + " dW_neigh")
        assert_close(gb, rb, tag + " db")
        if need_dx:
            assert_close(gX, rX, tag + " dX")


def test_symmetric_weights_no_bias_and_constant_input(B, G):
    """GCN's symmetric normalisation as the aggregation matrix (no CSC arrays needed), no bias, and a
    constant input whose A'X is computed by the first forward only: three steps give the same result."""
    rowptr, col, X, Ws, Wn, _, dY = case(62, 11, 64, 32, False)
    g = G.gcn_graph(rowptr, col)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, c, deg)
    rY = oracle.sage_forward(rp, c, val, X, Ws, Wn)
    rWs, rWn, _, rX = oracle.sage_backward(rp, c, val, X, Ws, Wn, dY)
    for steps, const in ((1, False), (3, True)):
        Y, gWs, gWn, gb, gX, info = run_sage(B, g, X, Ws, Wn, None, dY, True, False, schemes(B)["pf_sp_cache"],
                                             constant_input=const, steps=steps)
        assert info.cache == B.GNN_CACHE_AX and gb is None
        assert_close(Y, rY, "Y")
        assert_close(gWs, rWs, "dW_self")
        assert_close(gWn, rWn, "dW_neigh")
        assert_close(gX, rX, "dX")


def test_full_size_config2_shapes(B, G):
    """The bench graph (R-MAT 2^17) at one narrow and one wide output, AUTO plan, sampled rows of Y and dX
    and the whole weight gradients against the oracle."""
    rowptr, col, X, Ws, Wn, b, dY = case(63, 17, 128, 16, False)
    g = G.gcn_graph(rowptr, col, symmetric=False, aggregator=B.GNN_AGG_MEAN)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.aggregator_weights(rp, c, deg, "mean")
    Y, gWs, gWn, gb, gX, _ = run_sage(B, g, X, Ws, Wn, b, dY, True, False, dict())
    rY = oracle.sage_forward(rp, c, val, X, Ws, Wn, b)
    rWs, rWn, rb, rX = oracle.sage_backward(rp, c, val, X, Ws, Wn, dY)
    rows = np.random.default_rng(0).integers(0, X.shape[0], 4096)
    assert_close(Y[rows], rY[rows], "Y")
    assert_close(gX[rows], rX[rows], "dX")
    assert_close(gWs, rWs, "dW_self")
    assert_close(gWn, rWn, "dW_neigh")
    assert_close(gb, rb, "db")


def test_wrong_layer_kind_is_rejected(B, G):
    rowptr, col, X, Ws, Wn, b, dY = case(64, 8, 16, 16, False)
    g = G.gcn_graph(rowptr, col)
    plan = B.Plan(B.GNN_LAYER_GCN, g.n, g.nnz, 16, 16)
    ws = B.alloc(plan.info.workspace_bytes)
    Y = torch.zeros((g.n, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(B.GnnError):
        B.sage_layer_fwd(plan, g, dev(X), dev(Ws), dev(Wn), None, Y, None, ws)
