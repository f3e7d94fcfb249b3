// The plan object behind gnn_plan_t: the caller's description, the resolved scheme and
// buffer sizes, and whether a forward pass has filled the cache.
#pragma once

#include "common.h"

struct gnn_plan {
    gnn_plan_desc_t desc;
    gnn_plan_info_t info;
    bool cache_filled = false;
};

namespace gnn {

using Plan = ::gnn_plan;

// Byte offsets of the GAT cache blocks (in `cache`) and scratch blocks (in `workspace`).
// (size_t)-1 marks a block that does not exist in this variant.
struct GatLayout {
    size_t c_M, c_s, c_d, c_alpha, c_mask, cache_bytes;
    size_t w_M, w_s, w_d, w_alpha, w_stat, w_walk, w_spmm, w_gemm_nn;          // used by forward (and backward)
    size_t w_gy, w_sums, w_ds, w_dd, w_spmm_h, w_dM, w_red, w_gemm_tn, w_G;    // backward only (w_G: fused ELU)
    size_t w_fused, w_node;                                                    // fused edge passes: partials; per-node scratch
    size_t workspace_bytes;
};

GatLayout gat_layout(const Plan &p);
gnn_status_t plan_create(const gnn_plan_desc_t *desc, Plan **out);

gnn_status_t gcn_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *b, float *Y,
                         void *cache, void *workspace, hipStream_t st);
gnn_status_t gcn_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *Y,
                          const float *dY, float *dW, float *db, float *dX, void *cache, void *workspace,
                          hipStream_t st);
gnn_status_t gat_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *a_src,
                         const float *a_dst, const float *b, float *Y, void *cache, void *workspace, hipStream_t st);
gnn_status_t gat_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *W, const float *a_src,
                          const float *a_dst, const float *Y, const float *dY, float *dW, float *da_src,
                          float *da_dst, float *db, float *dX, void *cache, void *workspace, hipStream_t st);
gnn_status_t sage_forward(Plan &p, const gnn_graph_t &g, const float *X, const float *Ws, const float *Wn,
                          const float *b, float *Y, void *cache, void *workspace, hipStream_t st);
gnn_status_t sage_backward(Plan &p, const gnn_graph_t &g, const float *X, const float *Ws, const float *Wn,
                           const float *Y, const float *dY, float *dWs, float *dWn, float *db, float *dX,
                           void *cache, void *workspace, hipStream_t st);
double spmm_time_model_us(int64_t n, int64_t nnz, int f);

}  // namespace gnn
