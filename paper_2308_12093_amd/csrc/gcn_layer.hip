// GCN layer forward / backward as sequences of SpMM and GEMM launches, in the order
// the plan chose (Sec. 3.1; Fig. "Two schemes of computing the forward pass", Fig.
// "Alternative schemes of computing the backward pass", Fig. "GCN computation scheme
// using caching").  Host code: it only carves the workspace and enqueues kernels.
// The GraphSAGE layer (Sec. 3.1 "Generalizability") is the same chain plus a dense
// self term, added by the GEMM that follows or precedes the SpMM.
#include "plan.h"

namespace gnn {

namespace {

struct SparseView {            // a CSR view of A' or of A'^T
    const int32_t *ptr, *idx, *eidx;
    EdgeWeights w;
};

SparseView forward_view(const gnn_graph_t &g, int f) {
    return SparseView{g.csr_rowptr, g.csr_col, g.csr_erow, EdgeWeights{g.csr_val, nullptr, 1, f}};
}

// A'^T as a CSR matrix is the CSC arrays of A'; a symmetric A' is its own transpose.
SparseView transposed_view(const gnn_graph_t &g, int f) {
    if (g.symmetric) return forward_view(g, f);
    if (g.csc_val) return SparseView{g.csc_colptr, g.csc_row, g.csc_ecol, EdgeWeights{g.csc_val, nullptr, 1, f}};
    return SparseView{g.csc_colptr, g.csc_row, g.csc_ecol, EdgeWeights{g.csr_val, g.csc_perm, 1, f}};
}

gnn_status_t spmm(const gnn_graph_t &g, const SparseView &v, const float *B, int f, float *C, const float *bias,
                  int relu, void *ws, hipStream_t st) {
    return spmm_launch(g.n, g.nnz, v.ptr, v.idx, v.eidx, v.w, B, g.n, f, C, bias, relu, ws, st);
}

}  // namespace

gnn_status_t gcn_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *b, float *Y,
                         void *cache, void *workspace, hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, m = d.f_in, k = d.f_out;
    const float *bias = d.has_bias ? b : nullptr;
    Carver ws(workspace);
    if (p.info.order == GNN_ORDER_TRANSFORM_FIRST) {
        // T = X W, then Y = A' T (+ b, ReLU) fused into the SpMM write
        float *T = ws.take<float>((size_t)n * k);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, k));
        void *wt = ws.take<char>(gemm_workspace_bytes(0, 0, n, k, m));
        // a width that the SpMM runs on a padded operand: the GEMM writes T in that layout, where the SpMM looks for it
        int ldt = k;
        if (float *Tp = spmm_padded_operand(sp, g.csr_erow, n, d.nnz, k, &ldt)) T = Tp;
        GNN_TRY(gemm_launch(0, 0, n, k, m, X, W, T, nullptr, 0, wt, st, nullptr, 0, ldt));
        GNN_TRY(spmm(g, forward_view(g, k), T, k, Y, bias, d.fuse_relu, sp, st));
    } else {
        // P = A' X (kept in the cache slot when the plan caches it), then Y = P W (+ b, ReLU)
        const bool cached = p.info.cache == GNN_CACHE_AX;
        float *P = cached ? static_cast<float *>(cache) : ws.take<float>((size_t)n * m);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, m));
        void *wt = ws.take<char>(gemm_workspace_bytes(0, 0, n, k, m));
        // a constant input (promised by the caller) needs its A'X only once
        if (!(cached && d.constant_input && p.cache_filled))
            GNN_TRY(spmm(g, forward_view(g, m), X, m, P, nullptr, 0, sp, st));
        GNN_TRY(gemm_launch(0, 0, n, k, m, P, W, Y, bias, d.fuse_relu, wt, st));
        if (cached) p.cache_filled = true;
    }
    return GNN_OK;
}

gnn_status_t gcn_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *Y,
                          const float *dY, float *dW, float *db, float *dX, void *cache, void *workspace,
                          hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, m = d.f_in, k = d.f_out;
    const bool dx = d.need_input_grad != 0;
    Carver ws(workspace);

    // Gradient through the fused ReLU: G = dY .* [Y > 0].  When the only readers of G are the weight-gradient
    // product and the bias sum (split-propagate scheme without dX: the first layer of a network), they apply
    // the mask to dY as they load it and G is never written; otherwise one pass makes it.
    const bool mask_in_consumers = d.fuse_relu && p.info.bwd == GNN_BWD_SPLIT_PROPAGATE && !dx;
    const float *mask_y = mask_in_consumers ? Y : nullptr;
    const float *G = dY;
    float *Gm = d.fuse_relu ? ws.take<float>((size_t)n * k) : nullptr;   // carved either way: the layout is the plan's
    if (d.fuse_relu && !mask_in_consumers) {
        GNN_TRY(activation_grad_launch((int64_t)n * k, dY, Y, Gm, kActRelu, st));
        G = Gm;
    }
    if (d.has_bias) {                               // db = G^T 1
        void *red = ws.take<char>(colsum_workspace_bytes(n, k));
        GNN_TRY(colsum_launch(n, k, G, db, red, st, mask_y, kActRelu));
    }
    void *gemm_ws = ws.take<char>(gemm_workspace_bytes(1, 0, m, k, n));

    if (p.info.bwd == GNN_BWD_FUSED_PROPAGATE) {
        // H = A'^T G once; dW = X^T H; dX = H W^T
        float *H = ws.take<float>((size_t)n * k);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, k));
        GNN_TRY(spmm(g, transposed_view(g, k), G, k, H, nullptr, 0, sp, st));
        GNN_TRY(gemm_launch(1, 0, m, k, n, X, H, dW, nullptr, 0, gemm_ws, st));
        if (dx) GNN_TRY(gemm_launch(0, 1, n, m, k, H, W, dX, nullptr, 0, nullptr, st));
    } else {
        // dW = (A'X)^T G with A'X from the cache or recomputed; dX = A'^T (G W^T)
        const bool cached = p.info.cache == GNN_CACHE_AX;
        const float *P = static_cast<const float *>(cache);
        float *Pw = cached ? nullptr : ws.take<float>((size_t)n * m);
        float *U = dx ? ws.take<float>((size_t)n * m) : nullptr;
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, m));
        if (!cached) {
            GNN_TRY(spmm(g, forward_view(g, m), X, m, Pw, nullptr, 0, sp, st));
            P = Pw;
        }
        GNN_TRY(gemm_launch(1, 0, m, k, n, P, G, dW, nullptr, 0, gemm_ws, st, mask_y, kActRelu));
        if (dx) {
            const SparseView tv = transposed_view(g, m);
            int ldu = m;                                    // as in the forward pass: U written where the SpMM pads
            if (float *Up = spmm_padded_operand(sp, tv.eidx, n, d.nnz, m, &ldu)) U = Up;
            GNN_TRY(gemm_launch(0, 1, n, m, k, G, W, U, nullptr, 0, nullptr, st, nullptr, 0, ldu));
            GNN_TRY(spmm(g, tv, U, m, dX, nullptr, 0, sp, st));
        }
    }
    return GNN_OK;
}

// Y = X Ws + A' X Wn + b.  Aggregate first: one product over both operand pairs, [X | A'X] [Ws; Wn], writes Y
// once with bias and ReLU.  Transform first: the self term is a GEMM that adds to what the SpMM wrote.
gnn_status_t sage_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *Ws, const float *Wn,
                          const float *b, float *Y, void *cache, void *workspace, hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, m = d.f_in, k = d.f_out;
    const float *bias = d.has_bias ? b : nullptr;
    const int last = kActAccumulate | (d.fuse_relu ? kActRelu : 0);
    Carver ws(workspace);
    if (p.info.order == GNN_ORDER_TRANSFORM_FIRST) {
        float *T = ws.take<float>((size_t)n * k);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, k));
        void *wt = ws.take<char>(2 * gemm_workspace_bytes(0, 0, n, k, m));
        int ldt = k;
        if (float *Tp = spmm_padded_operand(sp, g.csr_erow, n, d.nnz, k, &ldt)) T = Tp;
        GNN_TRY(gemm_launch(0, 0, n, k, m, X, Wn, T, nullptr, 0, wt, st, nullptr, 0, ldt));
        GNN_TRY(spmm(g, forward_view(g, k), T, k, Y, nullptr, 0, sp, st));
        GNN_TRY(gemm_launch(0, 0, n, k, m, X, Ws, Y, bias, last, wt, st));
    } else {
        const bool cached = p.info.cache == GNN_CACHE_AX;
        float *P = cached ? static_cast<float *>(cache) : ws.take<float>((size_t)n * m);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, m));
        void *wt = ws.take<char>(2 * gemm_workspace_bytes(0, 0, n, k, m));
        if (!(cached && d.constant_input && p.cache_filled))
            GNN_TRY(spmm(g, forward_view(g, m), X, m, P, nullptr, 0, sp, st));
        GNN_TRY(gemm_launch(0, 0, n, k, m, X, Ws, Y, bias, d.fuse_relu, wt, st, nullptr, 0, 0, P, Wn));
        if (cached) p.cache_filled = true;
    }
    return GNN_OK;
}

gnn_status_t sage_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *Ws, const float *Wn,
                           const float *Y, const float *dY, float *dWs, float *dWn, float *db, float *dX,
                           void *cache, void *workspace, hipStream_t st) {
    const gnn_plan_desc_t &d = p.desc;
    const int n = d.n, m = d.f_in, k = d.f_out;
    const bool dx = d.need_input_grad != 0;
    Carver ws(workspace);

    // as in the GCN layer: without dX in the split-propagate scheme the masked gradient is only read by the two
    // weight-gradient products and the bias sum, which apply the mask as they load dY
    const bool mask_in_consumers = d.fuse_relu && p.info.bwd == GNN_BWD_SPLIT_PROPAGATE && !dx;
    const float *mask_y = mask_in_consumers ? Y : nullptr;
    const float *G = dY;
    float *Gm = d.fuse_relu ? ws.take<float>((size_t)n * k) : nullptr;
    if (d.fuse_relu && !mask_in_consumers) {
        GNN_TRY(activation_grad_launch((int64_t)n * k, dY, Y, Gm, kActRelu, st));
        G = Gm;
    }
    if (d.has_bias) {
        void *red = ws.take<char>(colsum_workspace_bytes(n, k));
        GNN_TRY(colsum_launch(n, k, G, db, red, st, mask_y, kActRelu));
    }
    void *gemm_ws = ws.take<char>(gemm_workspace_bytes(1, 0, m, k, n));
    GNN_TRY(gemm_launch(1, 0, m, k, n, X, G, dWs, nullptr, 0, gemm_ws, st, mask_y, kActRelu));     // dWs = X^T G

    if (p.info.bwd == GNN_BWD_FUSED_PROPAGATE) {
        // H = A'^T G once; dWn = X^T H; dX = G Ws^T + H Wn^T
        float *H = ws.take<float>((size_t)n * k);
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, k));
        GNN_TRY(spmm(g, transposed_view(g, k), G, k, H, nullptr, 0, sp, st));
        GNN_TRY(gemm_launch(1, 0, m, k, n, X, H, dWn, nullptr, 0, gemm_ws, st));
        if (dx) {
            GNN_TRY(gemm_launch(0, 1, n, m, k, G, Ws, dX, nullptr, 0, nullptr, st, nullptr, 0, 0, H, Wn));
        }
    } else {
        // dWn = (A'X)^T G with A'X from the cache or recomputed; dX = A'^T (G Wn^T) + G Ws^T
        const bool cached = p.info.cache == GNN_CACHE_AX;
        const float *P = static_cast<const float *>(cache);
        float *Pw = cached ? nullptr : ws.take<float>((size_t)n * m);
        float *U = dx ? ws.take<float>((size_t)n * m) : nullptr;
        void *sp = ws.take<char>(spmm_workspace_bytes(n, d.nnz, m));
        if (!cached) {
            GNN_TRY(spmm(g, forward_view(g, m), X, m, Pw, nullptr, 0, sp, st));
            P = Pw;
        }
        GNN_TRY(gemm_launch(1, 0, m, k, n, P, G, dWn, nullptr, 0, gemm_ws, st, mask_y, kActRelu));
        if (dx) {
            const SparseView tv = transposed_view(g, m);
            int ldu = m;
            if (float *Up = spmm_padded_operand(sp, tv.eidx, n, d.nnz, m, &ldu)) U = Up;
            GNN_TRY(gemm_launch(0, 1, n, m, k, G, Wn, U, nullptr, 0, nullptr, st, nullptr, 0, ldu));
            GNN_TRY(spmm(g, tv, U, m, dX, nullptr, 0, sp, st));
            GNN_TRY(gemm_launch(0, 1, n, m, k, G, Ws, dX, nullptr, kActAccumulate, nullptr, st));
        }
    }
    return GNN_OK;
}

}  // namespace gnn
