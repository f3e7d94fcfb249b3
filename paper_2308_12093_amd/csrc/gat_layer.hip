// GAT layer forward / backward (placeholder until the kernels land).
#include "plan.h"

namespace gnn {

gnn_status_t gat_forward(Plan &, const gnn_graph_t &, const float *, const float *, const float *, const float *,
                         const float *, float *, void *, void *, hipStream_t) {
    return GNN_ERR_UNSUPPORTED;
}

gnn_status_t gat_backward(Plan &, const gnn_graph_t &, const float *, const float *, const float *, const float *,
                          const float *, float *, float *, float *, float *, float *, void *, void *, hipStream_t) {
    return GNN_ERR_UNSUPPORTED;
}

gnn_status_t sddmm_launch(int, int, const int32_t *, const int32_t *, const float *, const float *, const float *, int,
                          int, float *, hipStream_t) {
    return GNN_ERR_UNSUPPORTED;
}

}  // namespace gnn
