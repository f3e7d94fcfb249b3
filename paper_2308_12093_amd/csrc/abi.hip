// extern "C" entry points: argument checks, then the internal launchers.
// Every check runs before the first launch, so a failing call has no side effect.
#include "plan.h"

using namespace gnn;

namespace {

hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

bool bad_align(const void *p) { return (reinterpret_cast<uintptr_t>(p) % kAlign) != 0; }

// cache / workspace of a layer call against what the plan reported
gnn_status_t check_buffers(const gnn_plan_t *plan, bool cache_used, const void *cache, size_t cache_bytes,
                           const void *workspace, size_t workspace_bytes) {
    if (!workspace || (cache_used && !cache)) return GNN_ERR_INVALID_ARG;
    if (bad_align(workspace) || (cache && bad_align(cache))) return GNN_ERR_INVALID_ARG;
    if (workspace_bytes < plan->info.workspace_bytes) return GNN_ERR_BUFFER_TOO_SMALL;
    if (cache_used && cache_bytes < plan->info.cache_bytes) return GNN_ERR_BUFFER_TOO_SMALL;
    return GNN_OK;
}

gnn_status_t check_graph(const gnn_plan_t *plan, const gnn_graph_t *g, bool need_val, bool need_transpose,
                         bool need_perm) {
    if (!g) return GNN_ERR_INVALID_ARG;
    if (g->n != plan->desc.n || g->nnz != plan->desc.nnz) return GNN_ERR_BAD_GRAPH;
    if (!g->csr_rowptr || (g->nnz > 0 && !g->csr_col)) return GNN_ERR_BAD_GRAPH;
    if (need_val && g->nnz > 0 && !g->csr_val) return GNN_ERR_BAD_GRAPH;
    if (need_transpose) {
        if (!g->csc_colptr || (g->nnz > 0 && !g->csc_row)) return GNN_ERR_BAD_GRAPH;
        if (g->nnz > 0 && need_perm && !g->csc_perm) return GNN_ERR_BAD_GRAPH;
    }
    return GNN_OK;
}

}  // namespace

extern "C" {

const char *gnn_status_string(gnn_status_t s) {
    switch (s) {
        case GNN_OK: return "ok";
        case GNN_ERR_INVALID_ARG: return "invalid argument";
        case GNN_ERR_BAD_GRAPH: return "graph does not match the plan or lacks required arrays";
        case GNN_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case GNN_ERR_STATE: return "backward needs a cache that no forward has filled";
        case GNN_ERR_UNSUPPORTED: return "unsupported shape";
        case GNN_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

gnn_status_t gnn_plan_create(const gnn_plan_desc_t *desc, gnn_plan_t **out) { return plan_create(desc, out); }

gnn_status_t gnn_plan_query(const gnn_plan_t *plan, gnn_plan_info_t *out) {
    if (!plan || !out) return GNN_ERR_INVALID_ARG;
    *out = plan->info;
    return GNN_OK;
}

void gnn_plan_destroy(gnn_plan_t *plan) { delete plan; }

gnn_status_t gnn_plan_reset_cache(gnn_plan_t *plan) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    plan->cache_filled = false;
    return GNN_OK;
}

double gnn_spmm_time_model_us(int64_t n, int64_t nnz, int32_t f) { return spmm_time_model_us(n, nnz, f); }

gnn_status_t gcn_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *b, float *Y, void *cache, size_t cache_bytes,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_GCN) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_graph(plan, graph, true, false, false));
    if (!X || !W || !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !b) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, plan->info.cache == GNN_CACHE_AX, cache, cache_bytes, workspace, workspace_bytes));
    if (plan->desc.n == 0) return GNN_OK;
    return gcn_forward(*plan, *graph, X, W, b, Y, cache, workspace, as_stream(hip_stream));
}

gnn_status_t gcn_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *Y, const float *dY, float *dW, float *db, float *dX,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_GCN) return GNN_ERR_INVALID_ARG;
    const bool cached = plan->info.cache == GNN_CACHE_AX;
    const bool needs_t = !graph || !graph->symmetric;
    const bool runs_spmm_t = plan->info.bwd == GNN_BWD_FUSED_PROPAGATE || plan->desc.need_input_grad;
    GNN_TRY(check_graph(plan, graph, true, needs_t && runs_spmm_t, graph && !graph->csc_val));
    if (!W || !dY || !dW) return GNN_ERR_INVALID_ARG;
    if (!cached && !X) return GNN_ERR_INVALID_ARG;
    if (plan->desc.fuse_relu && !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !db) return GNN_ERR_INVALID_ARG;
    if (plan->desc.need_input_grad && !dX) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, cached, cache, cache_bytes, workspace, workspace_bytes));
    if (cached && !plan->cache_filled) return GNN_ERR_STATE;
    if (plan->desc.n == 0) {
        // an empty graph has zero gradients; dW / db still have to be written (by a kernel of the library:
        // a memset node would not survive HIP graph capture of the call)
        hipStream_t st = as_stream(hip_stream);
        GNN_TRY(fill_zero_launch((int64_t)plan->desc.f_in * plan->desc.f_out, dW, st));
        if (plan->desc.has_bias) GNN_TRY(fill_zero_launch(plan->desc.f_out, db, st));
        return GNN_OK;
    }
    return gcn_backward(*plan, *graph, X, W, Y, dY, dW, db, dX, cache, workspace, as_stream(hip_stream));
}

gnn_status_t sage_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W_self,
                            const float *W_neigh, const float *b, float *Y, void *cache, size_t cache_bytes,
                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_SAGE) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_graph(plan, graph, true, false, false));
    if (!X || !W_self || !W_neigh || !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !b) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, plan->info.cache == GNN_CACHE_AX, cache, cache_bytes, workspace, workspace_bytes));
    if (plan->desc.n == 0) return GNN_OK;
    return sage_forward(*plan, *graph, X, W_self, W_neigh, b, Y, cache, workspace, as_stream(hip_stream));
}

gnn_status_t sage_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W_self,
                            const float *W_neigh, const float *Y, const float *dY, float *dW_self,
                            float *dW_neigh, float *db, float *dX, void *cache, size_t cache_bytes,
                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_SAGE) return GNN_ERR_INVALID_ARG;
    const bool cached = plan->info.cache == GNN_CACHE_AX;
    const bool needs_t = !graph || !graph->symmetric;
    const bool runs_spmm_t = plan->info.bwd == GNN_BWD_FUSED_PROPAGATE || plan->desc.need_input_grad;
    GNN_TRY(check_graph(plan, graph, true, needs_t && runs_spmm_t, graph && !graph->csc_val));
    if (!X || !W_self || !W_neigh || !dY || !dW_self || !dW_neigh) return GNN_ERR_INVALID_ARG;
    if (plan->desc.fuse_relu && !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !db) return GNN_ERR_INVALID_ARG;
    if (plan->desc.need_input_grad && !dX) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, cached, cache, cache_bytes, workspace, workspace_bytes));
    if (cached && !plan->cache_filled) return GNN_ERR_STATE;
    if (plan->desc.n == 0) {
        hipStream_t st = as_stream(hip_stream);
        const int64_t wc = (int64_t)plan->desc.f_in * plan->desc.f_out;
        GNN_TRY(fill_zero_launch(wc, dW_self, st));
        GNN_TRY(fill_zero_launch(wc, dW_neigh, st));
        if (plan->desc.has_bias) GNN_TRY(fill_zero_launch(plan->desc.f_out, db, st));
        return GNN_OK;
    }
    return sage_backward(*plan, *graph, X, W_self, W_neigh, Y, dY, dW_self, dW_neigh, db, dX, cache, workspace,
                         as_stream(hip_stream));
}

gnn_status_t gat_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *a_src, const float *a_dst, const float *b, float *Y,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_GAT) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_graph(plan, graph, false, false, false));
    if (!X || !W || !a_src || !a_dst || !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !b) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, plan->info.cache != GNN_CACHE_NONE, cache, cache_bytes, workspace, workspace_bytes));
    if (plan->desc.n == 0) return GNN_OK;
    return gat_forward(*plan, *graph, X, W, a_src, a_dst, b, Y, cache, workspace, as_stream(hip_stream));
}

gnn_status_t gat_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *a_src, const float *a_dst, const float *Y, const float *dY,
                           float *dW, float *da_src, float *da_dst, float *db, float *dX,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream) {
    if (!plan || plan->desc.layer != GNN_LAYER_GAT) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_graph(plan, graph, false, true, true));
    if (!X || !W || !a_src || !a_dst || !dY || !dW || !da_src || !da_dst) return GNN_ERR_INVALID_ARG;
    if (plan->desc.has_bias && !db) return GNN_ERR_INVALID_ARG;
    if (plan->desc.fuse_elu && !Y) return GNN_ERR_INVALID_ARG;
    if (plan->desc.need_input_grad && !dX) return GNN_ERR_INVALID_ARG;
    GNN_TRY(check_buffers(plan, plan->info.cache != GNN_CACHE_NONE, cache, cache_bytes, workspace, workspace_bytes));
    if (plan->info.cache != GNN_CACHE_NONE && !plan->cache_filled) return GNN_ERR_STATE;
    if (plan->desc.n == 0) {
        hipStream_t st = as_stream(hip_stream);
        const int64_t f = (int64_t)plan->desc.heads * plan->desc.f_out;
        GNN_TRY(fill_zero_launch((int64_t)plan->desc.f_in * f, dW, st));
        GNN_TRY(fill_zero_launch(f, da_src, st));
        GNN_TRY(fill_zero_launch(f, da_dst, st));
        if (plan->desc.has_bias) GNN_TRY(fill_zero_launch(f, db, st));
        return GNN_OK;
    }
    return gat_backward(*plan, *graph, X, W, a_src, a_dst, Y, dY, dW, da_src, da_dst, db, dX, cache, workspace,
                        as_stream(hip_stream));
}

// ---- preprocessing ---------------------------------------------------------------

size_t gnn_scan_workspace_bytes(int32_t n) { return scan_workspace_bytes(n > 0 ? n : 0); }

gnn_status_t gnn_add_self_loops_degree(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col,
                                       int32_t *rowptr_out, int32_t *col_out, int32_t *deg_out,
                                       int32_t *nnz_out_host, void *workspace, size_t workspace_bytes,
                                       void *hip_stream) {
    if (n < 0 || nnz < 0 || !rowptr || !rowptr_out || !col_out || !nnz_out_host || !workspace) return GNN_ERR_INVALID_ARG;
    if ((nnz > 0 && !col) || (n > 0 && !deg_out)) return GNN_ERR_INVALID_ARG;
    if ((int64_t)nnz + n > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    if (workspace_bytes < scan_workspace_bytes(n)) return GNN_ERR_BUFFER_TOO_SMALL;
    hipStream_t st = as_stream(hip_stream);
    GNN_TRY(add_self_loops_launch(n, nnz, rowptr, col, rowptr_out, col_out, deg_out, workspace, st));
    if (hipMemcpyAsync(nnz_out_host, rowptr_out + n, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return GNN_ERR_HIP;
    return hipStreamSynchronize(st) == hipSuccess ? GNN_OK : GNN_ERR_HIP;
}

gnn_status_t gnn_gcn_normalize(int32_t n, const int32_t *rowptr, const int32_t *col, const int32_t *deg,
                               float *val_out, void *hip_stream) {
    if (n < 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (n > 0 && (!deg || !col || !val_out)) return GNN_ERR_INVALID_ARG;
    return normalize_launch(n, rowptr, col, deg, val_out, GNN_AGG_GCN_SYM, 0.f, as_stream(hip_stream));
}

gnn_status_t gnn_aggregator_weights(gnn_aggregator_t kind, float eps, int32_t n, const int32_t *rowptr,
                                    const int32_t *col, const int32_t *deg, float *val_out, void *hip_stream) {
    if (kind != GNN_AGG_GCN_SYM && kind != GNN_AGG_MEAN && kind != GNN_AGG_GIN_SUM) return GNN_ERR_INVALID_ARG;
    if (n < 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (n > 0 && (!deg || !col || !val_out)) return GNN_ERR_INVALID_ARG;
    return normalize_launch(n, rowptr, col, deg, val_out, kind, eps, as_stream(hip_stream));
}

size_t gnn_transpose_workspace_bytes(int32_t n, int32_t nnz) {
    return transpose_workspace_bytes(n > 0 ? n : 0, nnz > 0 ? nnz : 0);
}

gnn_status_t gnn_csr_transpose(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col,
                               int32_t *colptr_out, int32_t *row_out, int32_t *perm_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (n < 0 || nnz < 0 || !rowptr || !colptr_out || !workspace) return GNN_ERR_INVALID_ARG;
    if (nnz > 0 && (!col || !row_out || !perm_out)) return GNN_ERR_INVALID_ARG;
    if (workspace_bytes < transpose_workspace_bytes(n, nnz)) return GNN_ERR_BUFFER_TOO_SMALL;
    if (bad_align(workspace)) return GNN_ERR_INVALID_ARG;
    return transpose_launch(n, nnz, rowptr, col, colptr_out, row_out, perm_out, workspace, as_stream(hip_stream));
}

gnn_status_t gnn_expand_ptr(int32_t n, int32_t nnz, const int32_t *ptr, int32_t *out, void *hip_stream) {
    if (n < 0 || nnz < 0 || !ptr || (nnz > 0 && !out)) return GNN_ERR_INVALID_ARG;
    return expand_ptr_launch(n, nnz, ptr, out, as_stream(hip_stream));
}

gnn_status_t gnn_gather_f32(int64_t count, const float *in, const int32_t *perm, float *out, void *hip_stream) {
    if (count < 0 || (count > 0 && (!in || !perm || !out))) return GNN_ERR_INVALID_ARG;
    return gather_f32_launch(count, in, perm, out, as_stream(hip_stream));
}

// ---- operators ----------------------------------------------------------------------

size_t gnn_spmm_workspace_bytes(int32_t n, int32_t nnz, int32_t f) {
    return spmm_workspace_bytes(n > 0 ? n : 0, nnz > 0 ? nnz : 0, f > 0 ? f : 1);
}

gnn_status_t gnn_spmm_csr(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col, const float *val,
                          const int32_t *erow, const float *B, int32_t f, float *C,
                          const float *bias, int32_t relu,
                          void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (n < 0 || nnz < 0 || f <= 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (relu != 0 && relu != 1) return GNN_ERR_INVALID_ARG;       // other activation codes are internal
    if (n > 0 && !C) return GNN_ERR_INVALID_ARG;
    if (nnz > 0 && (!col || !B)) return GNN_ERR_INVALID_ARG;
    if (erow && nnz > 0) {
        if (!workspace || bad_align(workspace)) return GNN_ERR_INVALID_ARG;
        if (workspace_bytes < spmm_workspace_bytes(n, nnz, f)) return GNN_ERR_BUFFER_TOO_SMALL;
    }
    return spmm_launch(n, nnz, rowptr, col, erow, EdgeWeights{val, nullptr, 1, f}, B, n, f, C, bias, relu, workspace,
                       as_stream(hip_stream));
}

gnn_status_t gnn_sddmm_csr(int32_t n, int32_t nnz, const int32_t *erow, const int32_t *col, const float *val,
                           const float *B, const float *Ct, int32_t heads, int32_t f, float *D,
                           void *hip_stream) {
    if (n < 0 || nnz < 0 || f <= 0 || heads <= 0) return GNN_ERR_INVALID_ARG;
    if (nnz > 0 && (!erow || !col || !B || !Ct || !D)) return GNN_ERR_INVALID_ARG;
    return sddmm_launch(n, nnz, erow, col, val, B, Ct, heads, f, D, as_stream(hip_stream));
}

size_t gnn_gat_aggregate_workspace_bytes(int32_t nnz, int32_t heads, int32_t f) {
    return gat_fused_workspace_bytes(nnz > 0 ? nnz : 0, heads, f);
}

gnn_status_t gnn_gat_aggregate_csr(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *erow,
                                   const int32_t *col, const float *M, const float *s, const float *d,
                                   int32_t heads, int32_t f, float leaky_slope, const float *bias, int32_t elu,
                                   float *Y, float *stat_out, void *workspace, size_t workspace_bytes,
                                   void *hip_stream) {
    if (n < 0 || nnz < 0 || heads <= 0 || f <= 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (n > 0 && (!Y || !stat_out)) return GNN_ERR_INVALID_ARG;
    if (nnz > 0 && (!erow || !col || !M || !s || !d || !workspace || bad_align(workspace))) return GNN_ERR_INVALID_ARG;
    if (!gat_fused_shape(n, nnz, heads, f) || !aligned16(M) || !aligned16(Y) || !aligned16(bias)) return GNN_ERR_UNSUPPORTED;
    if (nnz > 0 && workspace_bytes < gat_fused_workspace_bytes(nnz, heads, f)) return GNN_ERR_BUFFER_TOO_SMALL;
    return gat_fused_forward_launch(n, nnz, heads, f, rowptr, erow, col, M, s, d, leaky_slope, bias,
                                    elu ? kActElu : kActNone, Y, stat_out, workspace, as_stream(hip_stream));
}

size_t gnn_gemm_workspace_bytes(int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return kAlign;
    return gemm_workspace_bytes(trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K);
}

size_t gnn_hyb_workspace_bytes(int32_t n) { return n < 0 ? 0 : scan_workspace_bytes(n) + kAlign; }

gnn_status_t gnn_csr_hyb_count(int32_t n, const int32_t *rowptr, int32_t t, int32_t *rest_ptr_out,
                               int32_t *rest_nnz_out_host, int32_t *max_row_out_host,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (n < 0 || t < 0 || !rowptr || !rest_ptr_out || !workspace || bad_align(workspace)) return GNN_ERR_INVALID_ARG;
    if (workspace_bytes < gnn_hyb_workspace_bytes(n)) return GNN_ERR_BUFFER_TOO_SMALL;
    hipStream_t st = as_stream(hip_stream);
    int32_t *max_len = static_cast<int32_t *>(workspace);
    void *scan_ws = static_cast<char *>(workspace) + kAlign;
    GNN_TRY(hyb_count_launch(n, rowptr, t, rest_ptr_out, max_len, scan_ws, st));
    if (rest_nnz_out_host &&
        hipMemcpyAsync(rest_nnz_out_host, rest_ptr_out + n, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return GNN_ERR_HIP;
    if (max_row_out_host &&
        hipMemcpyAsync(max_row_out_host, max_len, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return GNN_ERR_HIP;
    return hipStreamSynchronize(st) == hipSuccess ? GNN_OK : GNN_ERR_HIP;
}

gnn_status_t gnn_csr_to_hyb(int32_t n, int32_t t, const int32_t *rowptr, const int32_t *col, const float *val,
                            const int32_t *rest_ptr, int32_t *ell_col, float *ell_val,
                            int32_t *coo_row, int32_t *coo_col, float *coo_val, void *hip_stream) {
    if (n < 0 || t < 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (n > 0 && t > 0 && (!ell_col || !ell_val)) return GNN_ERR_INVALID_ARG;
    if (rest_ptr && (!coo_row || !coo_col || !coo_val)) return GNN_ERR_INVALID_ARG;
    if (t == 0 && !rest_ptr) return GNN_ERR_INVALID_ARG;
    if ((int64_t)n * t / 256 >= INT32_MAX) return GNN_ERR_UNSUPPORTED;        // one thread per ELLPACK slot
    return hyb_fill_launch(n, t, rowptr, col, val, rest_ptr, ell_col, ell_val, coo_row, coo_col, coo_val,
                           as_stream(hip_stream));
}

gnn_status_t gnn_spmm_ell(int32_t n, int32_t t, const int32_t *ell_col, const float *ell_val,
                          const float *B, int32_t f, float *C, void *hip_stream) {
    if (n < 0 || t < 0 || f < 0) return GNN_ERR_INVALID_ARG;
    if (n == 0 || f == 0) return GNN_OK;
    if (!B || !C || (t > 0 && (!ell_col || !ell_val))) return GNN_ERR_INVALID_ARG;
    return spmm_ell_launch(n, t, ell_col, ell_val, B, f, C, as_stream(hip_stream));
}

gnn_status_t gnn_spmm_coo(int32_t n, int64_t nnz, const int32_t *row, const int32_t *col, const float *val,
                          const float *B, int32_t f, float *C, int32_t accumulate, void *hip_stream) {
    if (n < 0 || nnz < 0 || f < 0) return GNN_ERR_INVALID_ARG;
    if (n == 0 || f == 0) return GNN_OK;
    if (!B || !C || (nnz > 0 && (!row || !col))) return GNN_ERR_INVALID_ARG;
    hipStream_t st = as_stream(hip_stream);
    if (!accumulate) GNN_TRY(fill_zero_launch((int64_t)n * f, C, st));
    return spmm_coo_launch(nnz, row, col, val, B, f, C, st);
}

gnn_status_t gnn_spmm_hyb(int32_t n, int32_t t, const int32_t *ell_col, const float *ell_val,
                          int64_t rest_nnz, const int32_t *coo_row, const int32_t *coo_col, const float *coo_val,
                          const float *B, int32_t f, float *C, void *hip_stream) {
    GNN_TRY(gnn_spmm_ell(n, t, ell_col, ell_val, B, f, C, hip_stream));
    return gnn_spmm_coo(n, rest_nnz, coo_row, coo_col, coo_val, B, f, C, 1, hip_stream);
}

gnn_status_t gnn_gemm(int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K,
                      const float *A, const float *B, float *C, const float *bias, int32_t relu,
                      void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (M < 0 || N < 0 || K < 0) return GNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return GNN_OK;
    if (!C || (K > 0 && (!A || !B))) return GNN_ERR_INVALID_ARG;
    if (trans_a && trans_b) return GNN_ERR_UNSUPPORTED;
    if (relu & ~(GNN_GEMM_RELU | GNN_GEMM_ACCUMULATE)) return GNN_ERR_INVALID_ARG;
    if (trans_a && (relu & GNN_GEMM_ACCUMULATE)) return GNN_ERR_UNSUPPORTED;
    const size_t need = gnn_gemm_workspace_bytes(trans_a, trans_b, M, N, K);
    if (trans_a || !trans_b) {                          // only the A B^T form needs no scratch
        if (!workspace || bad_align(workspace)) return GNN_ERR_INVALID_ARG;
        if (workspace_bytes < need) return GNN_ERR_BUFFER_TOO_SMALL;
    }
    return gemm_launch(trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, B, C, bias, relu, workspace,
                       as_stream(hip_stream));
}

gnn_status_t gnn_softmax_xent(int32_t n, int32_t c, const float *Z, const int32_t *labels, float *dZ,
                              float *loss_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (n < 0 || c <= 0 || !loss_out) return GNN_ERR_INVALID_ARG;
    if (n > 0 && (!Z || !labels || !dZ || !workspace)) return GNN_ERR_INVALID_ARG;
    if (workspace_bytes < sizeof(float) * (size_t)ceil_div(n > 0 ? n : 1, 256)) return GNN_ERR_BUFFER_TOO_SMALL;
    return softmax_xent_launch(n, c, Z, labels, dZ, loss_out, workspace, as_stream(hip_stream));
}

gnn_status_t gnn_sum_squared_error(int64_t count, const float *Z, const float *T, float *dZ, float *loss_out,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (count < 0 || !loss_out || !workspace) return GNN_ERR_INVALID_ARG;
    if (count > 0 && (!Z || !T || !dZ)) return GNN_ERR_INVALID_ARG;
    if (workspace_bytes < 4096) return GNN_ERR_BUFFER_TOO_SMALL;
    return squared_error_launch(count, Z, T, dZ, loss_out, workspace, as_stream(hip_stream));
}

}  // extern "C"
