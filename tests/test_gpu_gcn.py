"""Parity of gcn_layer_fwd / gcn_layer_bwd with the fp64 oracle for every scheme, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_12093_amd import synth
from tests._util import assert_close, dev, host, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2308_12093_amd import binding
    return binding


@pytest.fixture(scope="module")
def G():
    from paper_2308_12093_amd import graphs
    return graphs


def schemes(B):
    return {
        "auto": dict(),
        "tf_fp": dict(order=B.GNN_ORDER_TRANSFORM_FIRST, bwd=B.GNN_BWD_FUSED_PROPAGATE, cache=B.GNN_CACHE_NONE),
        "pf_sp_nocache": dict(order=B.GNN_ORDER_PROPAGATE_FIRST, bwd=B.GNN_BWD_SPLIT_PROPAGATE, cache=B.GNN_CACHE_NONE),
        "pf_sp_cache": dict(order=B.GNN_ORDER_PROPAGATE_FIRST, bwd=B.GNN_BWD_SPLIT_PROPAGATE, cache=B.GNN_CACHE_AX),
        "pf_fp": dict(order=B.GNN_ORDER_PROPAGATE_FIRST, bwd=B.GNN_BWD_FUSED_PROPAGATE, cache=B.GNN_CACHE_NONE),
        "tf_sp": dict(order=B.GNN_ORDER_TRANSFORM_FIRST, bwd=B.GNN_BWD_SPLIT_PROPAGATE, cache=B.GNN_CACHE_NONE),
    }


def run_layer(B, g, X, W, b, dY, need_dx, relu, scheme, Y_for_mask=None):
    """One forward + backward through the C ABI.  Returns host arrays."""
    n, m = X.shape
    k = W.shape[1]
    plan = B.Plan(B.GNN_LAYER_GCN, g.n, g.nnz, m, k, need_input_grad=need_dx, has_bias=b is not None,
                  fuse_relu=relu, **scheme)
    ws = B.alloc(plan.info.workspace_bytes)
    cache = B.alloc(plan.info.cache_bytes) if plan.info.cache_bytes else None
    dX_, dW_, db_ = dev(X), dev(W), None if b is None else dev(b)
    Y = torch.full((n, k), float("nan"), dtype=torch.float32, device="cuda")
    B.gcn_layer_fwd(plan, g, dX_, dW_, db_, Y, cache, ws)
    torch.cuda.synchronize()
    ws.fill_(0xFF)                                             # backward must not rely on forward's scratch
    gW = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda")
    gb = None if b is None else torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
    gX = torch.full((n, m), float("nan"), dtype=torch.float32, device="cuda") if need_dx else None
    Ymask = None
    if relu:
        Ymask = Y if Y_for_mask is None else dev(Y_for_mask)
    x_arg = None if plan.info.cache == B.GNN_CACHE_AX else dX_    # with A'X cached the input is not needed
    B.gcn_layer_bwd(plan, g, x_arg, dW_, Ymask, dev(dY), gW, gb, gX, cache, ws)
    torch.cuda.synchronize()
    return host(Y), host(gW), None if gb is None else host(gb), None if gX is None else host(gX), plan.info


def oracle_layer(rp, c, val, X, W, b, dY, need_dx, relu, Y_for_mask=None):
    Y = oracle.gcn_forward(rp, c, val, X, W, b, relu)
    mask_src = None
    if relu:
        mask_src = Y_for_mask if Y_for_mask is not None else Y.astype(np.float32)
    dW, db, dX = oracle.gcn_backward(rp, c, val, X, W, dY, mask_src, need_dx)
    return Y, dW, db, dX


def check(B, G, rowptr, col, X, W, b, dY, need_dx, relu, scheme, symmetric=True, label=""):
    g = G.gcn_graph(rowptr, col, symmetric=symmetric)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, c, deg)
    # both sides take the ReLU sign decisions from the same float32 array: the oracle's forward output
    Ymask = oracle.gcn_forward(rp, c, val, X, W, b, True).astype(np.float32) if relu else None
    Y, gW, gb, gX, info = run_layer(B, g, X, W, b, dY, need_dx, relu, scheme, Ymask)
    rY, rW, rb, rX = oracle_layer(rp, c, val, X, W, b, dY, need_dx, relu, Ymask)
    assert_close(Y, rY, f"{label} Y")
    assert_close(gW, rW, f"{label} dW")
    if b is not None:
        assert_close(gb, rb, f"{label} db")
    if need_dx:
        assert_close(gX, rX, f"{label} dX")
    assert rel_fro(gW, rW) < 1e-5
    return info


@pytest.mark.parametrize("name", ["auto", "tf_fp", "pf_sp_nocache", "pf_sp_cache", "pf_fp", "tf_sp"])
@pytest.mark.parametrize("m,k", [(48, 16), (16, 48), (32, 32), (100, 47), (50, 70), (150, 200), (200, 150)])
def test_every_scheme_small_rmat(B, G, name, m, k):
    s = synth.streams(11)
    rowptr, col = synth.rmat_graph(11, 12, False, s["graph"], s["relabel"])
    n = rowptr.size - 1
    X, W = synth.normal(s["X"], n, m), synth.glorot_uniform(s["W"], (m, k), m, k)
    b, dY = synth.normal(s["b"], k), synth.normal(s["dY"], n, k)
    for need_dx in (True, False):
        for relu in (False, True):
            check(B, G, rowptr, col, X, W, b if relu else None, dY, need_dx, relu, schemes(B)[name],
                  label=f"{name} m={m} k={k} dx={need_dx} relu={relu}")


@pytest.mark.parametrize("name", ["auto", "tf_fp"])
@pytest.mark.parametrize("m,k", [(256, 256), (320, 264)])
def test_wide_layers_take_the_large_weight_gradient_tile(B, G, name, m, k):
    """F_in and F_out of 256 and more: dW = X^T H runs on the 128 x 128 tile of the fp64 split-K kernel."""
    s = synth.streams(17)
    rowptr, col = synth.rmat_graph(12, 10, False, s["graph"], s["relabel"])
    n = rowptr.size - 1
    X, W = synth.normal(s["X"], n, m), synth.glorot_uniform(s["W"], (m, k), m, k)
    b, dY = synth.normal(s["b"], k), synth.normal(s["dY"], n, k)
    check(B, G, rowptr, col, X, W, b, dY, True, True, schemes(B)[name], label=f"wide {name} m={m} k={k}")


@pytest.mark.parametrize("name", ["tf_fp", "pf_sp_nocache", "pf_sp_cache"])
def test_directed_graph_uses_the_transpose(B, G, name):
    s = synth.streams(12)
    rowptr, col = synth.rmat_graph(11, 10, True, s["graph"], s["relabel"])
    n = rowptr.size - 1
    X, W = synth.normal(s["X"], n, 24), synth.glorot_uniform(s["W"], (24, 40), 24, 40)
    check(B, G, rowptr, col, X, W, synth.normal(s["b"], 40), synth.normal(s["dY"], n, 40), True, False,
          schemes(B)[name], symmetric=False, label=f"directed {name}")


def test_config1_both_orderings(B, G):
    w = synth.config1()
    X, W, dY, b = w.tensors["X"], w.tensors["W16"], w.tensors["dY16"], None
    assert w.n == 2048 and w.col.size == 16384 and X.shape == (2048, 512) and W.shape == (512, 16)
    info = check(B, G, w.rowptr, w.col, X, W, b, dY, True, False, schemes(B)["auto"], label="cfg1 auto")
    assert info.order == B.GNN_ORDER_TRANSFORM_FIRST and info.bwd == B.GNN_BWD_FUSED_PROPAGATE
    for name in ("pf_sp_cache", "pf_sp_nocache"):
        for need_dx in (True, False):
            check(B, G, w.rowptr, w.col, X, W, b, dY, need_dx, False, schemes(B)[name], label=f"cfg1 {name}")


@pytest.mark.parametrize("k", [16, 128, 512])
def test_config2_full_size(B, G, k):
    """The benchmark workload itself, every element compared."""
    w = synth.config2(f_outs=(k,))
    X, W, dY = w.tensors["X"], w.tensors[f"W{k}"], w.tensors[f"dY{k}"]
    for name in ("auto", "tf_fp"):
        check(B, G, w.rowptr, w.col, X, W, None, dY, True, False, schemes(B)[name], label=f"cfg2 k={k} {name}")


def test_cached_backward_needs_a_forward_first(B, G):
    s = synth.streams(13)
    rowptr, col = synth.rmat_graph(8, 6, False, s["graph"], s["relabel"])
    g = G.gcn_graph(rowptr, col)
    plan = B.Plan(B.GNN_LAYER_GCN, g.n, g.nnz, 8, 16)
    assert plan.info.cache == B.GNN_CACHE_AX
    ws, cache = B.alloc(plan.info.workspace_bytes), B.alloc(plan.info.cache_bytes)
    t = lambda *shape: torch.zeros(shape, dtype=torch.float32, device="cuda")
    with pytest.raises(B.GnnError) as e:
        B.gcn_layer_bwd(plan, g, None, t(8, 16), None, t(g.n, 16), t(8, 16), None, t(g.n, 8), cache, ws)
    assert e.value.status == B.GNN_ERR_STATE


def test_constant_input_computes_the_cached_product_once(B, G):
    """A first layer whose input never changes (constant_input): forward fills the A'X cache once and
    later calls do not read X again until the cache is reset; results stay those of the oracle."""
    s = synth.streams(41)
    rowptr, col = synth.rmat_graph(10, 8, False, s["graph"], s["relabel"])
    n, m, k = rowptr.size - 1, 48, 16                          # k < m / 2: the rule alone would transform first
    X, X_other = synth.normal(s["X"], n, m), synth.normal(synth.substream(41, "X", 1), n, m)
    W1, W2 = synth.glorot_uniform(s["W"], (m, k), m, k), synth.glorot_uniform(s["W2"], (m, k), m, k)
    dY = synth.normal(s["dY"], n, k)
    g = G.gcn_graph(rowptr, col)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.gcn_normalize(rp, c, deg)
    plan = B.Plan(B.GNN_LAYER_GCN, g.n, g.nnz, m, k, need_input_grad=False, constant_input=True)
    assert (plan.info.order, plan.info.cache) == (B.GNN_ORDER_PROPAGATE_FIRST, B.GNN_CACHE_AX)
    ws, cache = B.alloc(plan.info.workspace_bytes), B.alloc(plan.info.cache_bytes)
    Y = torch.full((n, k), float("nan"), dtype=torch.float32, device="cuda")
    dW = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda")

    def step(x, w):
        B.gcn_layer_fwd(plan, g, dev(x), dev(w), None, Y, cache, ws)
        B.gcn_layer_bwd(plan, g, None, dev(w), None, dev(dY), dW, None, None, cache, ws)
        torch.cuda.synchronize()
        return host(Y), host(dW)

    y, dw = step(X, W1)                                        # iteration 1 fills the cache
    assert_close(y, oracle.gcn_forward(rp, c, val, X, W1), "iteration 1 Y")
    assert_close(dw, oracle.gcn_backward(rp, c, val, X, W1, dY, None, False)[0], "iteration 1 dW")
    y, dw = step(X_other, W2)                                  # new weights; the X argument is not read
    assert_close(y, oracle.gcn_forward(rp, c, val, X, W2), "iteration 2 Y (cached A'X)")
    assert_close(dw, oracle.gcn_backward(rp, c, val, X, W2, dY, None, False)[0], "iteration 2 dW")
    plan.reset_cache()
    y, dw = step(X_other, W2)                                  # after a reset the new input counts
    assert_close(y, oracle.gcn_forward(rp, c, val, X_other, W2), "after reset Y")
    assert_close(dw, oracle.gcn_backward(rp, c, val, X_other, W2, dY, None, False)[0], "after reset dW")


@pytest.mark.parametrize("kind,directed", [("mean", False), ("mean", True), ("gin", False), ("gin", True)])
@pytest.mark.parametrize("name", ["auto", "tf_fp", "pf_sp_cache"])
def test_mean_and_gin_aggregation_run_through_the_same_layer(B, G, kind, directed, name):
    """Other layers with the same chained product (Sec. 3.1 "Generalizability"): only the entry
    values differ, so the layer entry points, the orders and the cache are the ones of GCN.
    Mean weights (1 / deg_i) are not symmetric even on an undirected graph: backward goes through
    the CSC arrays."""
    s = synth.streams(51)
    rowptr, col = synth.rmat_graph(10, 8, directed, s["graph"], s["relabel"])
    n, m, k = rowptr.size - 1, 40, 24
    X, W = synth.normal(s["X"], n, m), synth.glorot_uniform(s["W"], (m, k), m, k)
    b, dY = synth.normal(s["b"], k), synth.normal(s["dY"], n, k)
    agg = dict(mean=B.GNN_AGG_MEAN, gin=B.GNN_AGG_GIN_SUM)[kind]
    eps = 0.3
    g = G.gcn_graph(rowptr, col, symmetric=not directed, aggregator=agg, eps=eps)
    assert g.c.symmetric == (0 if (directed or kind == "mean") else 1)
    rp, c, deg = oracle.add_self_loops_degree(rowptr, col)
    val = oracle.aggregator_weights(rp, c, deg, kind, eps)
    assert_close(host(g.val), val, f"{kind} weights", tol=1e-6)
    for need_dx in (True, False):
        Y, gW, gb, gX, _ = run_layer(B, g, X, W, b, dY, need_dx, False, schemes(B)[name])
        rY, rW, rb, rX = oracle_layer(rp, c, val, X, W, b, dY, need_dx, False)
        assert_close(Y, rY, f"{kind} {name} Y")
        assert_close(gW, rW, f"{kind} {name} dW")
        assert_close(gb, rb, f"{kind} {name} db")
        if need_dx:
            assert_close(gX, rX, f"{kind} {name} dX")


@pytest.mark.parametrize("n", [1, 2, 65])
def test_graph_without_edges_reduces_to_a_dense_layer(B, G, n):
    """Only the added self-loops remain: A' = I, so the layer is X W + b and its gradients are those of
    a dense layer (closed form, no oracle needed), whatever the scheme."""
    rowptr, col = np.zeros(n + 1, np.int32), np.zeros(0, np.int32)
    rng = np.random.default_rng(n)
    m, k = 12, 20
    X, W = rng.standard_normal((n, m), dtype=np.float32), rng.standard_normal((m, k), dtype=np.float32)
    b, dY = rng.standard_normal(k, dtype=np.float32), rng.standard_normal((n, k), dtype=np.float32)
    g = G.gcn_graph(rowptr, col)
    assert g.nnz == n and np.allclose(host(g.val), 1.0)
    X64, W64, dY64 = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)
    for name in ("tf_fp", "pf_sp_cache", "pf_sp_nocache"):
        Y, gW, gb, gX, _ = run_layer(B, g, X, W, b, dY, True, False, schemes(B)[name])
        assert_close(Y, X64 @ W64 + b, f"{name} Y")
        assert_close(gW, X64.T @ dY64, f"{name} dW")
        assert_close(gb, dY64.sum(axis=0), f"{name} db")
        assert_close(gX, dY64 @ W64.T, f"{name} dX")


def test_layer_calls_can_be_captured_in_a_hip_graph_and_replayed(B, G):
    """The layer entry points only enqueue kernels on the caller's stream, so a forward + backward
    can be recorded once and replayed; every replay (with eager work and synchronisations between
    them) must reproduce the eager result bit for bit."""
    s = synth.streams(61)
    rowptr, col = synth.rmat_graph(10, 8, False, s["graph"], s["relabel"])
    n, m, k = rowptr.size - 1, 64, 32
    g = G.gcn_graph(rowptr, col)
    X, W, dY = dev(synth.normal(s["X"], n, m)), dev(synth.glorot_uniform(s["W"], (m, k), m, k)), dev(synth.normal(s["dY"], n, k))
    for scheme in ("tf_fp", "pf_sp_cache"):
        plan = B.Plan(B.GNN_LAYER_GCN, g.n, g.nnz, m, k, **schemes(B)[scheme])
        ws = B.alloc(plan.info.workspace_bytes)
        cache = B.alloc(plan.info.cache_bytes) if plan.info.cache_bytes else None
        e = lambda *sh: torch.full(sh, float("nan"), dtype=torch.float32, device="cuda")
        Y, dW, dX = e(n, k), e(m, k), e(n, m)

        def step():
            B.gcn_layer_fwd(plan, g, X, W, None, Y, cache, ws)
            B.gcn_layer_bwd(plan, g, X, W, None, dY, dW, None, dX, cache, ws)

        step()
        torch.cuda.synchronize()
        eager = [host(t) for t in (Y, dW, dX)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                             # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for replay in range(3):
            for t in (Y, dW, dX):
                t.fill_(float("nan"))                          # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, ref, name in zip((Y, dW, dX), eager, ("Y", "dW", "dX")):
                assert np.array_equal(host(got), ref), f"{scheme} replay {replay}: {name}"
