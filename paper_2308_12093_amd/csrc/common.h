// Internal helpers shared by the host and device translation units of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gnn.h"

namespace gnn {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr size_t kAlign = 256;       // alignment of every carved workspace / cache block

// activation codes of the fused epilogues (the `relu` argument of the launchers: 0, 1 = the public values)
constexpr int kActNone = 0, kActRelu = 1, kActElu = 2;
// fp32 GEMM only, or-ed into its `relu` argument: add the product to what C already holds (before the activation)
constexpr int kActAccumulate = 4;
// set by the GEMM launcher itself for outputs beyond kStreamBytes: non-temporal stores
constexpr int kActStream = 8;
constexpr size_t kStreamBytes = (size_t)64 << 20;

static inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Carves consecutive aligned blocks out of one caller buffer.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T> T *take(size_t count) {
        T *r = reinterpret_cast<T *>(base + off);
        off += align_up(count * sizeof(T));
        return r;
    }
};

static inline gnn_status_t launch_status() {
    return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_HIP;
}

#define GNN_TRY(expr)                                  \
    do {                                               \
        gnn_status_t _s = (expr);                      \
        if (_s != GNN_OK) return _s;                   \
    } while (0)

// ---- sparse operators (spmm.hip) -------------------------------------------------
// How the weight of a stored entry is fetched.
struct EdgeWeights {
    const float *val;       // NULL: every weight is 1
    const int32_t *perm;    // NULL: slot e reads val[e...]; else val[perm[e]...]
    int32_t heads;          // 1: one weight per entry; >1: val is [nnz][heads], feature c uses head c / head_dim
    int32_t head_dim;
};

int spmm_segment_len(int64_t nnz, int f);
size_t spmm_workspace_bytes(int64_t n, int64_t nnz, int f);
// b_rows: rows of B (n when the column indices are node numbers), or 0 = unknown: then a width that is
// not a multiple of 4 is not run on a padded copy of B.  workspace: spmm_workspace_bytes(b_rows, nnz, f)
gnn_status_t spmm_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, const int32_t *erow,
                         EdgeWeights w, const float *B, long b_rows, int f, float *C, const float *bias, int relu,
                         void *workspace, hipStream_t st);
// The place inside `workspace` where such a call (one weight per entry) keeps its padded copy of B, rows *ld
// floats apart, or NULL when it makes none.  A caller that produces B itself may write it there in that layout
// (padding columns included, any finite value) and pass that address as B: the call then copies nothing.
float *spmm_padded_operand(void *workspace, const int32_t *erow, int64_t b_rows, int64_t nnz, int f, int *ld);

// ---- dense products (gemm.hip) ----------------------------------------------------
size_t gemm_workspace_bytes(int ta, int tb, int64_t M, int64_t N, int64_t K);
// b_mask (transposed-A form only): B is used as B .* act'(b_mask), the derivative of the activation
// b_mask_act (kActRelu, kActElu) taken from its output b_mask, an array of B's shape.
// ldc (plain products only): rows of C are ldc >= N floats apart, the columns in between written as zeros.
// A2, B2 (plain products only; shapes of A and B): C = op(A) op(B) + op(A2) op(B2) in one pass, one rounding
// chain; the untransposed-B form then needs a workspace of 2 x gemm_workspace_bytes.
gnn_status_t gemm_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, const float *B,
                         float *C, const float *bias, int relu, void *workspace, hipStream_t st,
                         const float *b_mask = nullptr, int b_mask_act = 0, int64_t ldc = 0,
                         const float *A2 = nullptr, const float *B2 = nullptr);

// ---- element-wise and reductions (elementwise.hip) ---------------------------------
// out = G * [Y > 0]
// out = G * act'(x) with the derivative taken from the activation's output Y (kActRelu or kActElu)
gnn_status_t activation_grad_launch(int64_t count, const float *G, const float *Y, float *out, int act, hipStream_t st);
// out[c] = sum_i G[i][c], deterministic two-stage; workspace colsum_workspace_bytes(n, f).
// With mask_y: the sum of G .* act'(mask_y) (mask_act: kActRelu or kActElu), as in activation_grad_launch.
size_t colsum_workspace_bytes(int64_t n, int f);
gnn_status_t colsum_launch(int64_t n, int f, const float *G, float *out, void *workspace, hipStream_t st,
                           const float *mask_y = nullptr, int mask_act = 0);
gnn_status_t squared_error_launch(int64_t count, const float *Z, const float *T, float *dZ, float *loss,
                                  void *workspace, hipStream_t st);
gnn_status_t softmax_xent_launch(int n, int c, const float *Z, const int32_t *labels, float *dZ, float *loss,
                                 void *workspace, hipStream_t st);

// ---- preprocessing (prep.hip) -------------------------------------------------------
size_t scan_workspace_bytes(int64_t n);
// in-place exclusive scan of `count` <= n + 1 integers; workspace scan_workspace_bytes(n)
gnn_status_t exclusive_scan_launch(int32_t *data, long count, void *workspace, hipStream_t st);
size_t transpose_workspace_bytes(int n, int nnz);
gnn_status_t add_self_loops_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, int32_t *rowptr_out,
                                   int32_t *col_out, int32_t *deg_out, void *workspace, hipStream_t st);
gnn_status_t normalize_launch(int n, const int32_t *rowptr, const int32_t *col, const int32_t *deg, float *val,
                              int kind, float eps, hipStream_t st);
gnn_status_t transpose_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, int32_t *colptr,
                              int32_t *row, int32_t *perm, void *workspace, hipStream_t st);
gnn_status_t expand_ptr_launch(int n, int nnz, const int32_t *ptr, int32_t *out, hipStream_t st);
gnn_status_t gather_f32_launch(int64_t count, const float *in, const int32_t *perm, float *out, hipStream_t st);

// ---- other storage formats (formats.hip) ----------------------------------------------
// rest_ptr [n + 1]: exclusive scan of max(0, row length - t); max_len_dev: one device word
gnn_status_t hyb_count_launch(int n, const int32_t *rowptr, int t, int32_t *rest_ptr, int32_t *max_len_dev,
                              void *scan_ws, hipStream_t st);
gnn_status_t hyb_fill_launch(int n, int t, const int32_t *rowptr, const int32_t *col, const float *val,
                             const int32_t *rest_ptr, int32_t *ell_col, float *ell_val, int32_t *coo_row,
                             int32_t *coo_col, float *coo_val, hipStream_t st);
gnn_status_t fill_zero_launch(int64_t count, float *p, hipStream_t st);
gnn_status_t spmm_ell_launch(int n, int t, const int32_t *ell_col, const float *ell_val, const float *B, int f,
                             float *C, hipStream_t st);
gnn_status_t spmm_coo_launch(int64_t nnz, const int32_t *row, const int32_t *col, const float *val, const float *B,
                             int f, float *C, hipStream_t st);

// ---- GAT kernels (gat.hip) -----------------------------------------------------------
int gat_segment_len(int64_t nnz, int h);
size_t gat_walker_workspace_bytes(int64_t nnz, int h);
gnn_status_t gat_node_attention_launch(int n, int h, int k, const float *M, const float *a_src, const float *a_dst,
                                       float *s, float *d, hipStream_t st);
// stat [n][h][2] (row max, sum of exponentials), alpha [nnz][h], mask [nnz][h] or NULL
gnn_status_t gat_edge_softmax_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                     const int32_t *col, const float *s, const float *d, float slope, float *stat,
                                     float *alpha, uint8_t *mask, void *workspace, hipStream_t st);
gnn_status_t gat_edge_stats_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                   const int32_t *col, const float *s, const float *d, float slope, float *stat,
                                   void *workspace, hipStream_t st);
gnn_status_t gat_edge_alpha_launch(int nnz, int h, const int32_t *erow, const int32_t *col, const float *s,
                                   const float *d, const float *stat, float slope, float *alpha, uint8_t *mask,
                                   hipStream_t st);
// gy [nnz][h]: g_alpha on entry, g_y on exit; sums [n][h][3] scratch; ds [n][h]; mask NULL: sign from s, d
gnn_status_t gat_edge_backward_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                      const int32_t *col, const float *alpha, const uint8_t *mask, const float *s,
                                      const float *d, float slope, float *gy, float *sums, float *ds,
                                      void *workspace, hipStream_t st);
gnn_status_t gat_add_rank1_launch(int n, int h, int k, const float *ds, const float *dd, const float *a_src,
                                  const float *a_dst, float *dM, hipStream_t st);
// da[p][c] = sum_i w[i][p] M[i][p][c]; workspace colsum_workspace_bytes(n, h*k)
gnn_status_t gat_attention_grad_launch(int n, int h, int k, const float *w, const float *M, float *da,
                                       void *workspace, hipStream_t st);
gnn_status_t sddmm_launch(int n, int nnz, const int32_t *erow, const int32_t *col, const float *val,
                          const float *B, const float *Ct, int heads, int f, float *D, hipStream_t st);

// ---- fused GAT edge passes (gat_fused.hip) -----------------------------------------------
bool gat_fused_shape(int64_t n, int64_t nnz, int h, int k);
size_t gat_fused_workspace_bytes(int64_t nnz, int h, int k);
// Y = act(softmax-weighted aggregation + bias), stat [n][h][2] = (row max, sum of exponentials)
gnn_status_t gat_fused_forward_launch(int n, int nnz, int h, int k, const int32_t *rowptr, const int32_t *erow,
                                      const int32_t *col, const float *M, const float *s, const float *d,
                                      float slope, const float *bias, int act, float *Y, float *stat, void *workspace,
                                      hipStream_t st);
// alpha / mask [q][h] in CSR order, or NULL: rebuilt from s, d.
// node: 4 n h floats of scratch.  Writes ds, dd [n][h] and the complete dM [n][h k].
gnn_status_t gat_fused_backward_launch(int n, int nnz, int h, int k, const int32_t *rowptr, const int32_t *erow,
                                       const int32_t *col, const int32_t *colptr, const int32_t *ecol,
                                       const int32_t *row, const int32_t *perm, const float *G, const float *M,
                                       const float *alpha, const uint8_t *mask, const float *s,
                                       const float *d, float slope, const float *a_src, const float *a_dst,
                                       float *node, float *ds, float *dd, float *dM, void *workspace, hipStream_t st);
// da_src[p][c] = sum_i ds[i][p] M[i][p][c] and da_dst likewise with dd, in one pass over M;
// workspace 2 * colsum_workspace_bytes(n, h*k)
gnn_status_t gat_attention_grad2_launch(int n, int h, int k, const float *ds, const float *dd, const float *M,
                                        float *da_src, float *da_dst, void *workspace, hipStream_t st);

}  // namespace gnn
