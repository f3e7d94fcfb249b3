"""CPU-only checks of the C-ABI library: it loads, exports what the header declares,
chooses schemes by the paper's tables and rejects bad arguments before any launch."""
import ctypes
import os
import subprocess
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

from paper_2308_12093_amd import binding as B  # noqa: E402


def header_functions():
    text = open(os.path.join(ROOT, "include", "gnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b((?:gnn|gcn|gat|sage)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported_and_bound():
    declared = header_functions()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(B.lib, name), name
        assert name in B.EXPORTS, name
    assert sorted(B.EXPORTS) == declared


def test_sage_plans_resolve_like_gcn_plans():
    """GraphSAGE runs SpMMs of the same widths as GCN, so every choice and buffer size is the same."""
    for m, k, dx in ((128, 16, True), (16, 128, True), (64, 64, False)):
        a = B.Plan(B.GNN_LAYER_GCN, 1000, 9000, m, k, need_input_grad=dx).info
        b = B.Plan(B.GNN_LAYER_SAGE, 1000, 9000, m, k, need_input_grad=dx).info
        assert (a.order, a.bwd, a.cache, a.cache_bytes, a.workspace_bytes) == \
               (b.order, b.bwd, b.cache, b.cache_bytes, b.workspace_bytes)
    with pytest.raises(B.GnnError):
        B.Plan(B.GNN_LAYER_SAGE, 1000, 9000, 8, 8, fuse_elu=True)
    with pytest.raises(B.GnnError):
        B.Plan(3, 1000, 9000, 8, 8)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 and as C++ with no HIP or torch include."""
    src = tmp_path / "use_header.c"
    src.write_text('#include "gnn.h"\nint main(void) { gnn_plan_desc_t d; gnn_graph_t g; (void)d; (void)g; return 0; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror"], ["g++", "-x", "c++", "-std=c++11", "-Wall", "-Werror"]):
        r = subprocess.run(cmd + ["-I", inc, "-c", str(src), "-o", str(tmp_path / "o.o")], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_status_strings():
    assert B.gnn_status_string(0) == "ok"
    for s in range(1, 7):
        assert B.gnn_status_string(s) not in ("ok", "unknown status")


def plan(m, k, dx, cache=B.GNN_CACHE_AUTO, order=B.GNN_ORDER_AUTO, bwd=B.GNN_BWD_AUTO, n=1000, nnz=9000, **kw):
    return B.Plan(B.GNN_LAYER_GCN, n, nnz, m, k, need_input_grad=dx, cache=cache, order=order, bwd=bwd, **kw)


TF, PF = B.GNN_ORDER_TRANSFORM_FIRST, B.GNN_ORDER_PROPAGATE_FIRST
FP, SP = B.GNN_BWD_FUSED_PROPAGATE, B.GNN_BWD_SPLIT_PROPAGATE


@pytest.mark.parametrize("m", [1, 7, 64, 128, 500])
def test_gcn_rule_without_caching(m):
    """Table "GCN schemes": forward TF iff k < m; backward FP iff k < 2m (with dX) / k < m (without)."""
    for k in sorted({1, m // 2, m - 1, m, m + 1, 2 * m - 1, 2 * m, 2 * m + 1, 5 * m} - {0}):
        for dx in (True, False):
            info = plan(m, k, dx, cache=B.GNN_CACHE_NONE).info
            assert info.order == (TF if k < m else PF), (m, k, dx)
            assert info.bwd == (FP if k < (2 * m if dx else m) else SP), (m, k, dx)
            assert info.cache == B.GNN_CACHE_NONE and info.cache_bytes == 0


@pytest.mark.parametrize("m", [2, 7, 64, 128, 500])
def test_gcn_rule_with_caching(m):
    """Table "GCN schemes with caching": TF+FP iff k < m (with dX) / k < m/2 (without); else PF+SP with cache."""
    for k in sorted({1, (m - 1) // 2, m // 2, m // 2 + 1, m - 1, m, m + 1, 3 * m} - {0}):
        for dx in (True, False):
            info = plan(m, k, dx).info
            small = (k < m) if dx else (2 * k < m)
            assert info.order == (TF if small else PF), (m, k, dx)
            assert info.bwd == (FP if small else SP), (m, k, dx)
            assert info.cache == (B.GNN_CACHE_NONE if small else B.GNN_CACHE_AX), (m, k, dx)


def test_observed_thresholds_at_128_input_features():
    """App. F: with 128 input features the schemes switch at 128 / 256 (no caching, without / with dX)
    and at 64 / 128 (caching, without / with dX)."""
    def first_switch(dx, cache):
        for k in (8, 16, 32, 64, 128, 256, 512, 1024):
            if plan(128, k, dx, cache=cache).info.bwd == SP:
                return k
    assert first_switch(False, B.GNN_CACHE_NONE) == 128
    assert first_switch(True, B.GNN_CACHE_NONE) == 256
    assert first_switch(False, B.GNN_CACHE_AUTO) == 64
    assert first_switch(True, B.GNN_CACHE_AUTO) == 128


def test_transients_and_spmm_widths_follow_the_tables():
    n, m = 1000, 128
    # TF + FP: nk; nk, two SpMMs of width k
    i = plan(m, 16, True).info
    assert (i.transient_fwd, i.transient_bwd, i.spmm_width_fwd, i.spmm_width_bwd) == (n * 16, n * 16, 16, 16)
    # PF + SP with cache, with dX: nm; nm, SpMMs of width m in each pass
    i = plan(m, 512, True).info
    assert (i.transient_fwd, i.transient_bwd, i.spmm_width_fwd, i.spmm_width_bwd) == (n * m, n * m, m, m)
    assert i.cache_bytes >= 4 * n * m and i.cache_bytes < 4 * n * m + 256
    # ... without dX: nm; 0 and no SpMM in backward
    i = plan(m, 512, False).info
    assert (i.transient_fwd, i.transient_bwd, i.spmm_width_bwd) == (n * m, 0, 0)
    # split-propagate without cache: two SpMMs of width m, 2nm transients
    i = plan(m, 512, True, cache=B.GNN_CACHE_NONE).info
    assert (i.bwd, i.transient_bwd, i.spmm_width_bwd) == (SP, 2 * n * m, 2 * m)


def test_forced_schemes_and_invalid_combinations():
    i = plan(128, 16, True, order=PF, bwd=SP).info
    assert (i.order, i.bwd, i.cache) == (PF, SP, B.GNN_CACHE_AX)
    i = plan(128, 16, True, order=PF, bwd=SP, cache=B.GNN_CACHE_NONE).info
    assert (i.order, i.bwd, i.cache) == (PF, SP, B.GNN_CACHE_NONE)
    i = plan(128, 512, True, order=TF, bwd=FP).info
    assert (i.order, i.bwd, i.cache) == (TF, FP, B.GNN_CACHE_NONE)
    with pytest.raises(B.GnnError) as e:
        plan(128, 512, True, order=TF, cache=B.GNN_CACHE_AX)      # A'X does not exist in transform-first
    assert e.value.status == B.GNN_ERR_INVALID_ARG
    for bad in (dict(m=0, k=4), dict(m=4, k=0), dict(m=4, k=4, n=-1)):
        with pytest.raises(B.GnnError):
            plan(bad.pop("m"), bad.pop("k"), True, **bad)
    with pytest.raises(B.GnnError):
        plan(4, 4, True, cache=B.GNN_CACHE_GAT_FEAT)


def test_gat_cache_sizes():
    """Table "GAT caching": 4nhk, 4nh(k+2), 4nhk + 5qh bytes (plus alignment padding per block)."""
    n, q, h, k = 1000, 9000, 8, 8
    want = {B.GNN_CACHE_NONE: 0, B.GNN_CACHE_GAT_FEAT: 4 * n * h * k,
            B.GNN_CACHE_GAT_FEAT_NODEATT: 4 * n * h * (k + 2), B.GNN_CACHE_GAT_FEAT_EDGE: 4 * n * h * k + 5 * q * h}
    for variant, size in want.items():
        info = B.Plan(B.GNN_LAYER_GAT, n, q, 256, k, heads=h, cache=variant).info
        assert size <= info.cache_bytes <= size + 3 * 256, (variant, info.cache_bytes, size)
        assert info.cache == variant
    assert B.Plan(B.GNN_LAYER_GAT, n, q, 256, k, heads=h).info.cache == B.GNN_CACHE_GAT_FEAT_EDGE
    # the calibrated choice: what is fastest on this machine (alpha rebuilt from the node values)
    assert B.Plan(B.GNN_LAYER_GAT, n, q, 256, k, heads=h, selection=B.GNN_SELECT_CALIBRATED).info.cache == \
        B.GNN_CACHE_GAT_FEAT_NODEATT


def test_layer_calls_reject_bad_arguments_before_any_launch():
    p = plan(8, 4, True, n=10, nnz=30)
    g = B.gnn_graph_t(10, 30, 256, 256, 256, None, None, None, None, None, None, 1)
    null = ctypes.c_void_p(None)
    one = ctypes.c_void_p(256)
    ws = p.info.workspace_bytes
    bufs = (null, 0, one, ws, null)                       # cache, cache_bytes, workspace, workspace_bytes, stream
    # NULL X
    assert B.lib.gcn_layer_fwd(p.handle, ctypes.byref(g), null, one, null, one, *bufs) == B.GNN_ERR_INVALID_ARG
    # misaligned workspace
    assert B.lib.gcn_layer_fwd(p.handle, ctypes.byref(g), one, one, null, one, null, 0, ctypes.c_void_p(260), ws,
                               null) == B.GNN_ERR_INVALID_ARG
    # graph that does not match the plan
    g2 = B.gnn_graph_t(11, 30, 256, 256, 256, None, None, None, None, None, None, 1)
    assert B.lib.gcn_layer_fwd(p.handle, ctypes.byref(g2), one, one, null, one, *bufs) == B.GNN_ERR_BAD_GRAPH
    # GCN needs edge values
    g3 = B.gnn_graph_t(10, 30, 256, 256, None, None, None, None, None, None, None, 1)
    assert B.lib.gcn_layer_fwd(p.handle, ctypes.byref(g3), one, one, null, one, *bufs) == B.GNN_ERR_BAD_GRAPH
    # backward on a directed graph without CSC arrays
    g4 = B.gnn_graph_t(10, 30, 256, 256, 256, None, None, None, None, None, None, 0)
    assert B.lib.gcn_layer_bwd(p.handle, ctypes.byref(g4), one, one, null, one, one, null, one, *bufs) == B.GNN_ERR_BAD_GRAPH
    # missing dX although the plan needs it
    assert B.lib.gcn_layer_bwd(p.handle, ctypes.byref(g), one, one, null, one, one, null, null, *bufs) == B.GNN_ERR_INVALID_ARG
    # a GAT call on a GCN plan
    assert B.lib.gat_layer_fwd(p.handle, ctypes.byref(g), one, one, one, one, null, one, *bufs) == B.GNN_ERR_INVALID_ARG


def test_layer_calls_reject_buffers_smaller_than_the_plan_reports():
    """Every layer call takes the byte sizes of cache and workspace and checks them before any launch."""
    null, one = ctypes.c_void_p(None), ctypes.c_void_p(256)
    sym = B.gnn_graph_t(10, 30, 256, 256, 256, 256, None, None, None, None, None, 1)
    full = B.gnn_graph_t(10, 30, 256, 256, 256, 256, 256, 256, 256, 256, 256, 0)
    small = B.GNN_ERR_BUFFER_TOO_SMALL
    # GCN, propagate-first with the A'X cache
    p = plan(8, 16, True, n=10, nnz=30)
    ws, cb = p.info.workspace_bytes, p.info.cache_bytes
    assert p.info.cache == B.GNN_CACHE_AX and cb >= 4 * 10 * 8 and ws > 0
    fwd = lambda *bufs: B.lib.gcn_layer_fwd(p.handle, ctypes.byref(sym), one, one, null, one, *bufs, null)
    assert fwd(one, cb, one, ws - 1) == small
    assert fwd(one, cb - 1, one, ws) == small
    assert fwd(null, cb, one, ws) == B.GNN_ERR_INVALID_ARG        # the plan caches: the buffer is required
    bwd = lambda *bufs: B.lib.gcn_layer_bwd(p.handle, ctypes.byref(sym), null, one, null, one, one, null, one, *bufs, null)
    assert bwd(one, cb, one, ws - 1) == small
    assert bwd(one, cb - 1, one, ws) == small
    assert bwd(one, cb, one, ws) == B.GNN_ERR_STATE               # sizes fine: only the missing forward remains
    # a plan without cache ignores the cache arguments
    p2 = plan(8, 4, True, n=10, nnz=30)
    assert p2.info.cache == B.GNN_CACHE_NONE
    assert B.lib.gcn_layer_fwd(p2.handle, ctypes.byref(sym), one, one, null, one, null, 0, one,
                               p2.info.workspace_bytes - 1, null) == small
    # GraphSAGE
    ps = B.Plan(B.GNN_LAYER_SAGE, 10, 30, 8, 16)
    assert B.lib.sage_layer_fwd(ps.handle, ctypes.byref(sym), one, one, one, null, one, one, ps.info.cache_bytes, one,
                                ps.info.workspace_bytes - 1, null) == small
    assert B.lib.sage_layer_bwd(ps.handle, ctypes.byref(sym), one, one, one, null, one, one, one, null, one, one,
                                ps.info.cache_bytes - 1, one, ps.info.workspace_bytes, null) == small
    # GAT, every caching variant
    for variant in (B.GNN_CACHE_NONE, B.GNN_CACHE_GAT_FEAT, B.GNN_CACHE_GAT_FEAT_NODEATT, B.GNN_CACHE_GAT_FEAT_EDGE):
        pg = B.Plan(B.GNN_LAYER_GAT, 10, 30, 8, 4, heads=2, cache=variant)
        ws, cb = pg.info.workspace_bytes, pg.info.cache_bytes
        c = one if cb else null
        gf = lambda *bufs: B.lib.gat_layer_fwd(pg.handle, ctypes.byref(full), one, one, one, one, null, one, *bufs, null)
        gb = lambda *bufs: B.lib.gat_layer_bwd(pg.handle, ctypes.byref(full), one, one, one, one, null, one, one, one,
                                               one, null, one, *bufs, null)
        assert gf(c, cb, one, ws - 1) == small and gb(c, cb, one, ws - 1) == small
        if cb:
            assert gf(c, cb - 1, one, ws) == small and gb(c, cb - 1, one, ws) == small
            assert gb(c, cb, one, ws) == B.GNN_ERR_STATE


def test_backward_before_forward_with_cached_plan_is_a_state_error():
    p = plan(8, 16, True, n=10, nnz=30)
    assert p.info.cache == B.GNN_CACHE_AX
    g = B.gnn_graph_t(10, 30, 256, 256, 256, None, None, None, None, None, None, 1)
    null, one = ctypes.c_void_p(None), ctypes.c_void_p(256)
    st = B.lib.gcn_layer_bwd(p.handle, ctypes.byref(g), null, one, null, one, one, null, one, one, p.info.cache_bytes,
                             one, p.info.workspace_bytes, null)
    assert st == B.GNN_ERR_STATE


def test_operator_calls_check_sizes():
    null, one = ctypes.c_void_p(None), ctypes.c_void_p(256)
    need = B.gnn_spmm_workspace_bytes(100, 1000, 64)
    assert need >= 2 * (1000 // 256) * 64 * 4
    st = B.lib.gnn_spmm_csr(100, 1000, one, one, one, one, one, 64, one, null, 0, one, need - 1, null)
    assert st == B.GNN_ERR_BUFFER_TOO_SMALL
    assert B.lib.gnn_spmm_csr(100, 1000, one, one, one, one, one, 0, one, null, 0, one, need, null) == B.GNN_ERR_INVALID_ARG
    # the activation argument takes 0 or 1 only (the library's other epilogue codes are internal)
    for relu in (2, 4, -1):
        assert B.lib.gnn_spmm_csr(100, 1000, one, one, one, one, one, 64, one, null, relu, one, need, null) == B.GNN_ERR_INVALID_ARG
    assert B.lib.gnn_gemm(1, 1, 4, 4, 4, one, one, one, null, 0, null, 0, null) == B.GNN_ERR_UNSUPPORTED
    assert B.lib.gnn_gemm(0, 0, -1, 4, 4, one, one, one, null, 0, null, 0, null) == B.GNN_ERR_INVALID_ARG
    tw = B.gnn_transpose_workspace_bytes(100, 1000)
    assert B.lib.gnn_csr_transpose(100, 1000, one, one, one, one, one, one, tw - 1, null) == B.GNN_ERR_BUFFER_TOO_SMALL
    # the fused GAT aggregation: head widths, alignment and the sizes its 32-bit gather offsets can address
    def aggregate(n, nnz, heads, f, M=one, bias=null, ws_bytes=1 << 30):
        return B.lib.gnn_gat_aggregate_csr(n, nnz, one, one, one, M, one, one, heads, f, 0.2, bias, 0, one, one, one,
                                           ws_bytes, null)
    for heads, f in ((2, 6), (1, 3), (2, 12), (1, 512)):
        assert aggregate(100, 1000, heads, f) == B.GNN_ERR_UNSUPPORTED
    assert aggregate(100, 1000, 2, 8, M=ctypes.c_void_p(260)) == B.GNN_ERR_UNSUPPORTED        # M not 16-byte aligned
    assert aggregate(100, 1000, 2, 8, bias=ctypes.c_void_p(260)) == B.GNN_ERR_UNSUPPORTED
    assert aggregate(1 << 24, 1000, 2, 8) == B.GNN_ERR_UNSUPPORTED                            # node numbers of 24 bits
    assert aggregate(1 << 23, 1000, 8, 64) == B.GNN_ERR_UNSUPPORTED                           # M of 16 GiB
    assert aggregate(1 << 20, 1 << 30, 8, 8) == B.GNN_ERR_UNSUPPORTED                         # nnz * heads = 2^33
    assert aggregate(100, 1000, 2, 8, ws_bytes=B.gnn_gat_aggregate_workspace_bytes(1000, 2, 8) - 1) == B.GNN_ERR_BUFFER_TOO_SMALL


# ---- calibrated selection and constant inputs (host logic) --------------------------------
def model_us(n, nnz, f):
    """The documented time model, evaluated here from the text of the header."""
    import math
    dense_mb = 4.0 * n * f / 1e6
    c = 0.32 if dense_mb <= 70.0 else min(0.53, 0.32 + 0.045 * math.log2(dense_mb / 70.0))
    return 12.0 + nnz * max(13.0, c * f) * 1e-6


def golden_times():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "spmm_times_mi355x.txt")):
        if line.strip() and not line.startswith("#"):
            n, nnz, f, us = line.split()
            rows.append((int(n), int(nnz), int(f), float(us)))
    return rows


def test_time_model_matches_its_documentation_and_the_measurements_it_was_fitted_to():
    """The stored file holds measured times of this library's own SpMM (timing data that a cost model was fitted
    to, not expected values of any computation): the check is that the model still describes them within 25-30 %,
    nothing that decides whether a result is correct."""
    for n, nnz, f, us in golden_times():
        got = B.gnn_spmm_time_model_us(n, nnz, f)
        assert got == pytest.approx(model_us(n, nnz, f), rel=1e-12)
        assert 0.75 * us <= got <= 1.3 * us, (n, nnz, f, us, got)
    assert B.gnn_spmm_time_model_us(0, 0, 16) == 0.0
    # monotone in the width, flat at the per-entry floor
    t = [B.gnn_spmm_time_model_us(131072, 1841460, f) for f in (8, 16, 32, 64, 128, 256)]
    assert t[0] == t[1] == t[2] and t[2] < t[3] < t[4] < t[5]


CAL = dict(selection=B.GNN_SELECT_CALIBRATED, n=131072, nnz=1841460)


def test_calibrated_selection_moves_the_crossovers_where_spmm_time_is_flat():
    FP, SP = B.GNN_BWD_FUSED_PROPAGATE, B.GNN_BWD_SPLIT_PROPAGATE
    # without dX the rule flips at k = m / 2 = 64; two narrow SpMMs cost more than half a wide one
    for k, rule, cal in ((32, TF, TF), (48, TF, TF), (60, TF, PF), (64, PF, PF)):
        assert plan(128, k, False, n=131072, nnz=1841460).info.order == rule
        assert plan(128, k, False, **CAL).info.order == cal
    # m = 64: a width-64 SpMM is cheaper than two at the floor, whatever k
    assert plan(64, 16, False, n=131072, nnz=1841460).info.order == TF
    p = plan(64, 16, False, **CAL)
    assert (p.info.order, p.info.bwd, p.info.cache) == (PF, SP, B.GNN_CACHE_AX)
    # the small graph of cfg1 (m = 512, k = 16, no dX): one launch pair less wins, as measured
    p = plan(512, 16, False, selection=B.GNN_SELECT_CALIBRATED, n=2048, nnz=18432)
    assert (p.info.order, p.info.cache) == (PF, B.GNN_CACHE_AX)
    assert plan(512, 16, True, selection=B.GNN_SELECT_CALIBRATED, n=2048, nnz=18432).info.order == TF
    # with dX both schemes run two SpMMs: same choice as the rule away from the floor
    for m, k in ((128, 64), (128, 256), (512, 128), (128, 512)):
        assert plan(m, k, True, **CAL).info.order == plan(m, k, True, n=131072, nnz=1841460).info.order
    # no caching, backward with dX: one SpMM of width 64 beats two of width 16 (rule: 64 >= 2 * 16 -> split)
    assert plan(16, 64, True, cache=B.GNN_CACHE_NONE, n=131072, nnz=1841460).info.bwd == SP
    assert plan(16, 64, True, cache=B.GNN_CACHE_NONE, **CAL).info.bwd == FP
    with pytest.raises(B.GnnError):
        plan(16, 16, True, selection=7)


def test_chosen_scheme_has_the_smallest_modelled_spmm_time():
    n, nnz = 131072, 1841460
    t = lambda f: B.gnn_spmm_time_model_us(n, nnz, f)
    for m in (16, 64, 128, 512):
        for k in (8, 16, 48, 64, 128, 256, 1024):
            for dx in (False, True):
                p = plan(m, k, dx, **CAL)
                cost = {TF: 2 * t(k), PF: t(m) + (t(m) if dx else 0.0)}
                assert cost[p.info.order] <= min(cost.values()) + 1e-9, (m, k, dx)


def test_constant_input_makes_the_cached_scheme_free_in_forward():
    SP = B.GNN_BWD_SPLIT_PROPAGATE
    for m, k in ((512, 16), (128, 8), (16, 16), (64, 512)):
        p = plan(m, k, False, constant_input=True)
        assert (p.info.order, p.info.bwd, p.info.cache) == (PF, SP, B.GNN_CACHE_AX), (m, k)
    # with dX the cached scheme still pays one SpMM of width m per iteration against two of width k
    assert plan(512, 16, True, constant_input=True).info.order == TF        # 2 * 16 < 512
    assert plan(128, 64, True, constant_input=True).info.order == PF        # 2 * 64 >= 128
    assert plan(128, 64, True).info.order == TF
    # no cache allowed: nothing to reuse
    assert plan(512, 16, False, constant_input=True, cache=B.GNN_CACHE_NONE).info.order == TF
    p = plan(128, 64, False, constant_input=True)
    p.reset_cache()
    with pytest.raises(B.GnnError):
        B.Plan(B.GNN_LAYER_GAT, 100, 900, 16, 8, heads=2, constant_input=True)
    with pytest.raises(B.GnnError):
        plan(16, 16, True, fuse_elu=True)
    assert B.Plan(B.GNN_LAYER_GAT, 100, 900, 16, 8, heads=2, fuse_elu=True).info.workspace_bytes > \
        B.Plan(B.GNN_LAYER_GAT, 100, 900, 16, 8, heads=2).info.workspace_bytes
