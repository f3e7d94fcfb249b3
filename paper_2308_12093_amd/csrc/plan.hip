// Scheme selection (Sec. 3.1, Tables "GCN schemes" and "GCN schemes with caching";
// Sec. 3.2 / Table "GAT caching") and the sizes that follow from it.  Host code only.
#include "plan.h"

#include <cmath>
#include <new>

namespace gnn {

namespace {

bool valid_enum(int v, int lo, int hi) { return v >= lo && v <= hi; }

// Cost of one SpMM of dense width f as the selection sees it: the width itself under the
// paper's rule (Sec. 3.1 takes SpMM time to be proportional to it), the fitted time of this
// library's kernel on an MI355X under the calibrated selection.
double spmm_cost(const gnn_plan_desc_t &d, int64_t f) {
    return d.selection == GNN_SELECT_CALIBRATED ? spmm_time_model_us(d.n, d.nnz, (int)f) : (double)f;
}

gnn_status_t resolve_gcn(Plan &p) {
    const gnn_plan_desc_t &d = p.desc;
    const int64_t m = d.f_in, k = d.f_out;
    const bool dx = d.need_input_grad != 0;
    if (d.cache != GNN_CACHE_AUTO && d.cache != GNN_CACHE_NONE && d.cache != GNN_CACHE_AX) return GNN_ERR_INVALID_ARG;
    const bool allow_cache = d.cache != GNN_CACHE_NONE;
    // The schemes differ only in their SpMMs (Tables "GCN schemes", "GCN schemes with caching"):
    //   transform-first forward  one of width k      propagate-first forward  one of width m
    //   fused-propagate backward one of width k      split-propagate backward  A'X (width m, unless
    //                                                cached) and, with dX, A'^T (G Theta^T) (width m)
    // With cost = width the comparisons below are the usage conditions printed in the tables
    // (ties go to propagate-first / split-propagate, as "k >= m" does there).
    const double ck = spmm_cost(d, k), cm = spmm_cost(d, m);
    const bool reuse = allow_cache && d.constant_input;           // A'X of a constant input is computed once
    const double cached_tf_fp_cost = 2 * ck;
    const double cached_pf_sp_cost = (reuse ? 0.0 : cm) + (dx ? cm : 0.0);
    const bool cached_tf_fp = cached_tf_fp_cost < cached_pf_sp_cost;
    const bool nocache_fwd_tf = ck < cm;
    const bool nocache_bwd_fp = ck < (dx ? 2 * cm : cm);

    gnn_order_t order = d.order;
    gnn_bwd_t bwd = d.bwd;
    if (order == GNN_ORDER_AUTO && bwd == GNN_BWD_AUTO) {
        if (allow_cache) {
            order = cached_tf_fp ? GNN_ORDER_TRANSFORM_FIRST : GNN_ORDER_PROPAGATE_FIRST;
            bwd = cached_tf_fp ? GNN_BWD_FUSED_PROPAGATE : GNN_BWD_SPLIT_PROPAGATE;
        } else {
            order = nocache_fwd_tf ? GNN_ORDER_TRANSFORM_FIRST : GNN_ORDER_PROPAGATE_FIRST;
            bwd = nocache_bwd_fp ? GNN_BWD_FUSED_PROPAGATE : GNN_BWD_SPLIT_PROPAGATE;
        }
    } else {
        if (order == GNN_ORDER_AUTO)
            order = (bwd == GNN_BWD_SPLIT_PROPAGATE && allow_cache) ? GNN_ORDER_PROPAGATE_FIRST
                    : (nocache_fwd_tf ? GNN_ORDER_TRANSFORM_FIRST : GNN_ORDER_PROPAGATE_FIRST);
        if (bwd == GNN_BWD_AUTO)
            bwd = (order == GNN_ORDER_PROPAGATE_FIRST && allow_cache) ? GNN_BWD_SPLIT_PROPAGATE
                  : (nocache_bwd_fp ? GNN_BWD_FUSED_PROPAGATE : GNN_BWD_SPLIT_PROPAGATE);
    }
    // A'X exists only in the propagate-first forward and is used only by the split-propagate backward
    const bool can_cache = order == GNN_ORDER_PROPAGATE_FIRST && bwd == GNN_BWD_SPLIT_PROPAGATE;
    if (d.cache == GNN_CACHE_AX && !can_cache) return GNN_ERR_INVALID_ARG;
    p.info.order = order;
    p.info.bwd = bwd;
    p.info.cache = (allow_cache && can_cache) ? GNN_CACHE_AX : GNN_CACHE_NONE;
    return GNN_OK;
}

void size_gcn(Plan &p) {
    const gnn_plan_desc_t &d = p.desc;
    const int64_t n = d.n, q = d.nnz, m = d.f_in, k = d.f_out;
    const bool dx = d.need_input_grad != 0;
    const bool tf = p.info.order == GNN_ORDER_TRANSFORM_FIRST;
    const bool fp = p.info.bwd == GNN_BWD_FUSED_PROPAGATE;
    const bool cached = p.info.cache == GNN_CACHE_AX;
    const size_t fl = sizeof(float);

    p.info.cache_bytes = cached ? align_up((size_t)n * m * fl) : 0;

    // forward
    size_t fwd = gemm_workspace_bytes(0, 0, n, k, m);
    if (d.layer == GNN_LAYER_SAGE) fwd *= 2;               // both weights transposed for the one product that uses both
    if (tf) {
        fwd += align_up((size_t)n * k * fl) + spmm_workspace_bytes(n, q, (int)k);
        p.info.transient_fwd = n * k;
        p.info.spmm_width_fwd = k;
    } else {
        if (!cached) fwd += align_up((size_t)n * m * fl);
        fwd += spmm_workspace_bytes(n, q, (int)m);
        p.info.transient_fwd = n * m;
        p.info.spmm_width_fwd = m;
    }
    // backward
    size_t bwd = 0;
    if (d.fuse_relu) bwd += align_up((size_t)n * k * fl);
    if (d.has_bias) bwd += colsum_workspace_bytes(n, (int)k);
    bwd += gemm_workspace_bytes(1, 0, m, k, n);
    if (fp) {
        bwd += align_up((size_t)n * k * fl) + spmm_workspace_bytes(n, q, (int)k);
        p.info.transient_bwd = n * k;
        p.info.spmm_width_bwd = k;
    } else {
        int64_t tr = 0, width = 0;
        if (!cached) { bwd += align_up((size_t)n * m * fl); tr += n * m; width += m; }
        if (dx) { bwd += align_up((size_t)n * m * fl); tr += n * m; width += m; }
        bwd += spmm_workspace_bytes(n, q, (int)m);
        p.info.transient_bwd = tr;
        p.info.spmm_width_bwd = width;
    }
    p.info.workspace_bytes = (fwd > bwd ? fwd : bwd) + kAlign;
}

gnn_status_t resolve_gat(Plan &p) {
    const gnn_plan_desc_t &d = p.desc;
    gnn_cache_t c = d.cache;
    // Sec. 4.2 finds the variant that keeps the edge weights fastest; on an MI355X, with the fused edge passes,
    // rebuilding alpha from four floats per node beats reading five bytes per entry and head, and the
    // variant that keeps the node attention values is the fastest measured
    if (c == GNN_CACHE_AUTO)
        c = d.selection == GNN_SELECT_CALIBRATED ? GNN_CACHE_GAT_FEAT_NODEATT : GNN_CACHE_GAT_FEAT_EDGE;
    if (c != GNN_CACHE_NONE && c != GNN_CACHE_GAT_FEAT && c != GNN_CACHE_GAT_FEAT_NODEATT &&
        c != GNN_CACHE_GAT_FEAT_EDGE)
        return GNN_ERR_INVALID_ARG;
    if (d.order != GNN_ORDER_AUTO && d.order != GNN_ORDER_TRANSFORM_FIRST) return GNN_ERR_INVALID_ARG;
    if (d.bwd != GNN_BWD_AUTO) return GNN_ERR_INVALID_ARG;
    p.info.order = GNN_ORDER_TRANSFORM_FIRST;                      // attention is computed from X Theta
    p.info.bwd = GNN_BWD_FUSED_PROPAGATE;
    p.info.cache = c;
    return GNN_OK;
}

}  // namespace

// Fitted to this library's entry-balanced SpMM on an MI355X (R-MAT graphs, 2^11 .. 2^22 nodes):
// a fixed cost of the two launches, then per entry the larger of a floor (index traffic and
// one cache line per gathered row, reached below ~32 columns) and a per-column cost that
// grows once the dense operand no longer fits the caches.
double spmm_time_model_us(int64_t n, int64_t nnz, int f) {
    if (n <= 0 || nnz <= 0 || f <= 0) return 0.0;
    const double dense_mb = 4.0 * (double)n * f / 1e6;
    double c = 0.32;                                               // ps per entry and column
    if (dense_mb > 70.0) c += 0.045 * std::log2(dense_mb / 70.0);
    if (c > 0.53) c = 0.53;
    const double per_entry_ps = c * f > 13.0 ? c * f : 13.0;
    return 12.0 + (double)nnz * per_entry_ps * 1e-6;
}

GatLayout gat_layout(const Plan &p) {
    const gnn_plan_desc_t &d = p.desc;
    const size_t n = d.n, q = d.nnz, h = d.heads, k = d.f_out, f = h * k, m = d.f_in, fl = sizeof(float);
    GatLayout L{};
    const gnn_cache_t c = p.info.cache;
    // cache blocks, in the documented order
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    L.c_M = L.c_s = L.c_d = L.c_alpha = L.c_mask = (size_t)-1;
    if (c != GNN_CACHE_NONE) L.c_M = take(n * f * fl);
    if (c == GNN_CACHE_GAT_FEAT_NODEATT) { L.c_s = take(n * h * fl); L.c_d = take(n * h * fl); }
    if (c == GNN_CACHE_GAT_FEAT_EDGE) { L.c_alpha = take(q * h * fl); L.c_mask = take(q * h); }
    L.cache_bytes = off;
    // workspace blocks: whatever is not cached, plus backward scratch
    off = 0;
    L.w_M = L.w_s = L.w_d = L.w_alpha = (size_t)-1;
    if (L.c_M == (size_t)-1) L.w_M = take(n * f * fl);
    if (L.c_s == (size_t)-1) { L.w_s = take(n * h * fl); L.w_d = take(n * h * fl); }
    if (L.c_alpha == (size_t)-1) L.w_alpha = take(q * h * fl);
    L.w_stat = take(n * h * 2 * fl);
    L.w_walk = take(gat_walker_workspace_bytes(q, (int)h));
    L.w_spmm = take(spmm_workspace_bytes(n, q, (int)f));
    L.w_gemm_nn = take(gemm_workspace_bytes(0, 0, n, f, m));
    L.w_gy = take(q * h * fl);
    L.w_sums = take(n * h * 3 * fl);
    L.w_ds = take(n * h * fl);
    L.w_dd = take(n * h * fl);
    L.w_spmm_h = take(spmm_workspace_bytes(0, q, (int)h));        // its dense operand has q rows: never padded
    L.w_dM = take(n * f * fl);
    L.w_red = take(2 * colsum_workspace_bytes(n, (int)f));
    L.w_gemm_tn = take(gemm_workspace_bytes(1, 0, m, f, n));
    L.w_G = d.fuse_elu ? take(n * f * fl) : (size_t)-1;
    L.w_fused = take(gat_fused_workspace_bytes(q, (int)h, (int)k));
    L.w_node = take(n * h * 4 * fl);
    L.workspace_bytes = off + kAlign;
    return L;
}

gnn_status_t plan_create(const gnn_plan_desc_t *desc, Plan **out) {
    if (!desc || !out) return GNN_ERR_INVALID_ARG;
    const gnn_plan_desc_t &d = *desc;
    if (!valid_enum(d.layer, GNN_LAYER_GCN, GNN_LAYER_SAGE) || !valid_enum(d.order, 0, 2) ||
        !valid_enum(d.bwd, 0, 2) || !valid_enum(d.cache, 0, 5))
        return GNN_ERR_INVALID_ARG;
    if (d.n < 0 || d.nnz < 0 || d.f_in <= 0 || d.f_out <= 0) return GNN_ERR_INVALID_ARG;
    if (!valid_enum(d.selection, GNN_SELECT_PAPER_RULE, GNN_SELECT_CALIBRATED)) return GNN_ERR_INVALID_ARG;
    if (d.layer != GNN_LAYER_GAT && d.fuse_elu) return GNN_ERR_INVALID_ARG;
    if (d.layer == GNN_LAYER_GAT && d.constant_input) return GNN_ERR_INVALID_ARG;
    Plan *p = new (std::nothrow) Plan();
    if (!p) return GNN_ERR_INVALID_ARG;
    p->desc = d;
    p->info = gnn_plan_info_t{};
    gnn_status_t s;
    if (d.layer != GNN_LAYER_GAT) {                       // GCN and SAGE: same schemes, same buffers
        p->desc.heads = 1;
        s = resolve_gcn(*p);
        if (s == GNN_OK) size_gcn(*p);
    } else {
        if (d.heads <= 0 || d.heads > 64 || d.fuse_relu) { delete p; return GNN_ERR_INVALID_ARG; }
        if ((int64_t)d.heads * d.f_out > (1 << 20)) { delete p; return GNN_ERR_UNSUPPORTED; }
        s = resolve_gat(*p);
        if (s == GNN_OK) {
            const GatLayout L = gat_layout(*p);
            p->info.cache_bytes = L.cache_bytes;
            p->info.workspace_bytes = L.workspace_bytes;
            const int64_t f = (int64_t)d.heads * d.f_out;
            p->info.transient_fwd = (int64_t)d.n * f;
            p->info.transient_bwd = (int64_t)d.n * f;
            p->info.spmm_width_fwd = f;
            p->info.spmm_width_bwd = f;
        }
    }
    if (s != GNN_OK) { delete p; return s; }
    *out = p;
    return GNN_OK;
}

}  // namespace gnn
