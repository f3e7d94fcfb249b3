// GAT layer forward / backward (Sec. "GAT Forward Pass", "GAT Backward Pass") as a
// sequence of kernel launches, with the caching variants of Table "GAT caching":
// whatever the plan's variant keeps (M; M, s, d; M, alpha, mask) is written to the
// cache by forward and read by backward, everything else is rebuilt in backward.
// The edge phase runs as three fused passes (gat_fused.hip) when the head width allows it
// (whole float4s per head, a power of two of them, 16-byte aligned rows), else as separate
// kernels per step (gat.hip, spmm.hip).  Host code: it only carves buffers and enqueues kernels.
#include "plan.h"

namespace gnn {

namespace {

struct Buffers {
    float *M, *s, *d, *alpha, *stat;
    uint8_t *mask;                 // NULL unless the variant caches it
};

template <typename T> T *at(void *base, size_t off) {
    return off == (size_t)-1 ? nullptr : reinterpret_cast<T *>(static_cast<char *>(base) + off);
}

Buffers pick_buffers(const GatLayout &L, void *cache, void *ws) {
    Buffers b;
    b.M = L.c_M != (size_t)-1 ? at<float>(cache, L.c_M) : at<float>(ws, L.w_M);
    b.s = L.c_s != (size_t)-1 ? at<float>(cache, L.c_s) : at<float>(ws, L.w_s);
    b.d = L.c_d != (size_t)-1 ? at<float>(cache, L.c_d) : at<float>(ws, L.w_d);
    b.alpha = L.c_alpha != (size_t)-1 ? at<float>(cache, L.c_alpha) : at<float>(ws, L.w_alpha);
    b.mask = at<uint8_t>(cache, L.c_mask);
    b.stat = at<float>(ws, L.w_stat);
    return b;
}

}  // namespace

gnn_status_t gat_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *a_src,
                         const float *a_dst, const float *b, float *Y, void *cache, void *workspace, hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, q = d.nnz, m = d.f_in, h = d.heads, k = d.f_out, f = h * k;
    if (!g.csr_erow && q > 0) return GNN_ERR_BAD_GRAPH;
    const GatLayout L = gat_layout(p);
    const Buffers B = pick_buffers(L, cache, workspace);

    // M = X Theta; s, d per node and head (App. B)
    GNN_TRY(gemm_launch(0, 0, n, f, m, X, W, B.M, nullptr, 0, at<char>(workspace, L.w_gemm_nn), st));
    GNN_TRY(gat_node_attention_launch(n, h, k, B.M, a_src, a_dst, B.s, B.d, st));
    const float *bias = d.has_bias ? b : nullptr;
    const int act = d.fuse_elu ? kActElu : kActNone;
    if (gat_fused_shape(n, q, h, k) && aligned16(Y) && aligned16(bias)) {
        // logits, LeakyReLU, row softmax and the weighted aggregation in one pass over the entries
        GNN_TRY(gat_fused_forward_launch(n, q, h, k, g.csr_rowptr, g.csr_erow, g.csr_col, B.M, B.s, B.d, d.leaky_slope,
                                         bias, act, Y, B.stat, at<char>(workspace, L.w_fused), st));
        // only the variant that keeps the edge weights materialises them
        if (p.info.cache == GNN_CACHE_GAT_FEAT_EDGE)
            GNN_TRY(gat_edge_alpha_launch(q, h, g.csr_erow, g.csr_col, B.s, B.d, B.stat, d.leaky_slope, B.alpha, B.mask, st));
    } else {
        // alpha = row softmax of LeakyReLU(s_i + d_j)
        GNN_TRY(gat_edge_softmax_launch(n, q, h, g.csr_rowptr, g.csr_erow, g.csr_col, B.s, B.d, d.leaky_slope, B.stat,
                                        B.alpha, B.mask, at<char>(workspace, L.w_walk), st));
        // Y_i = sum_e alpha_e M_j (+ b): SpMM with one weight per entry and head
        GNN_TRY(spmm_launch(n, q, g.csr_rowptr, g.csr_col, g.csr_erow, EdgeWeights{B.alpha, nullptr, h, k}, B.M, n, f, Y,
                            bias, act, at<char>(workspace, L.w_spmm), st));
    }
    p.cache_filled = true;
    return GNN_OK;
}

gnn_status_t gat_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *a_src,
                          const float *a_dst, const float *Y, const float *dY_in, float *dW, float *da_src,
                          float *da_dst, float *db, float *dX, void *cache, void *workspace, hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, q = d.nnz, m = d.f_in, h = d.heads, k = d.f_out, f = h * k;
    if ((!g.csr_erow || !g.csc_ecol) && q > 0) return GNN_ERR_BAD_GRAPH;
    const GatLayout L = gat_layout(p);
    const Buffers B = pick_buffers(L, cache, workspace);
    const gnn_cache_t variant = p.info.cache;

    // rebuild what the variant did not keep
    if (variant == GNN_CACHE_NONE)
        GNN_TRY(gemm_launch(0, 0, n, f, m, X, W, B.M, nullptr, 0, at<char>(workspace, L.w_gemm_nn), st));
    if (variant == GNN_CACHE_NONE || variant == GNN_CACHE_GAT_FEAT)
        GNN_TRY(gat_node_attention_launch(n, h, k, B.M, a_src, a_dst, B.s, B.d, st));
    const bool fused = gat_fused_shape(n, q, h, k) && aligned16(dY_in) && aligned16(a_src) && aligned16(a_dst);
    // the fused passes rebuild alpha per entry from per-node values; the separate kernels need the array
    if (variant != GNN_CACHE_GAT_FEAT_EDGE && !fused)
        GNN_TRY(gat_edge_softmax_launch(n, q, h, g.csr_rowptr, g.csr_erow, g.csr_col, B.s, B.d, d.leaky_slope, B.stat,
                                        B.alpha, nullptr, at<char>(workspace, L.w_walk), st));

    // gradient through the fused ELU, from the layer's output
    const float *dY = dY_in;
    if (d.fuse_elu) {
        float *G = at<float>(workspace, L.w_G);
        GNN_TRY(activation_grad_launch((int64_t)n * f, dY_in, Y, G, kActElu, st));
        dY = G;
    }

    float *gy = at<float>(workspace, L.w_gy), *sums = at<float>(workspace, L.w_sums);
    float *ds = at<float>(workspace, L.w_ds), *dd = at<float>(workspace, L.w_dd), *dM = at<float>(workspace, L.w_dM);

    if (d.has_bias) GNN_TRY(colsum_launch(n, f, dY, db, at<char>(workspace, L.w_red), st));
    if (fused) {
        // row pass: SDDMM folded into the row sums (ds, t); column pass: dd and dM = A^T G + ds a_src + dd a_dst
        const bool cached = variant == GNN_CACHE_GAT_FEAT_EDGE;
        GNN_TRY(gat_fused_backward_launch(n, q, h, k, g.csr_rowptr, g.csr_erow, g.csr_col, g.csc_colptr, g.csc_ecol,
                                          g.csc_row, g.csc_perm, dY, B.M, cached ? B.alpha : nullptr,
                                          cached ? B.mask : nullptr, B.s, B.d, d.leaky_slope, a_src, a_dst,
                                          at<float>(workspace, L.w_node), ds, dd, dM, at<char>(workspace, L.w_fused), st));
    } else {
        // dL/dalpha on the pattern: g_alpha_e = <G_i, M_j> per head (SDDMM)
        GNN_TRY(sddmm_launch(n, q, g.csr_erow, g.csr_col, nullptr, dY, B.M, h, k, gy, st));
        // softmax and LeakyReLU backward: g_y per entry, ds per node
        GNN_TRY(gat_edge_backward_launch(n, q, h, g.csr_rowptr, g.csr_erow, g.csr_col, B.alpha, B.mask, B.s, B.d,
                                         d.leaky_slope, gy, sums, ds, at<char>(workspace, L.w_walk), st));
        // dd_j = sum over column j of g_y: a row sum over the CSC arrays, gathering g_y rows through perm
        GNN_TRY(spmm_launch(n, q, g.csc_colptr, g.csc_perm, g.csc_ecol, EdgeWeights{nullptr, nullptr, 1, h}, gy, 0, h, dd,
                            nullptr, 0, at<char>(workspace, L.w_spmm_h), st));
        // dM = A^T G (weights alpha through perm) + ds a_src + dd a_dst
        GNN_TRY(spmm_launch(n, q, g.csc_colptr, g.csc_row, g.csc_ecol, EdgeWeights{B.alpha, g.csc_perm, h, k}, dY, n, f, dM,
                            nullptr, 0, at<char>(workspace, L.w_spmm), st));
        GNN_TRY(gat_add_rank1_launch(n, h, k, ds, dd, a_src, a_dst, dM, st));
    }
    // da_src = M^T ds, da_dst = M^T dd, one pass over M
    GNN_TRY(gat_attention_grad2_launch(n, h, k, ds, dd, B.M, da_src, da_dst, at<char>(workspace, L.w_red), st));
    // dTheta = X^T dM, dX = dM Theta^T
    GNN_TRY(gemm_launch(1, 0, m, f, n, X, dM, dW, nullptr, 0, at<char>(workspace, L.w_gemm_tn), st));
    if (d.need_input_grad) GNN_TRY(gemm_launch(0, 1, n, m, f, dM, W, dX, nullptr, 0, nullptr, st));
    return GNN_OK;
}

}  // namespace gnn
