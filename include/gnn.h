/*
 * gnn.h - C ABI of the MI355X (gfx950) GCN / GAT layer library.
 *
 * The library computes forward and backward passes of GCN and GAT layers
 * with adaptive operator reordering and caching (arXiv 2308.12093, Sec. 3).
 *
 * General rules, valid for every entry point below
 * ------------------------------------------------
 *  - Pointers named in a "device" position are DEVICE pointers (HIP global
 *    memory); they are borrowed for the duration of the enqueued work and are
 *    never freed or retained by the library.  gnn_plan_desc_t, gnn_plan_info_t,
 *    gnn_graph_t themselves are HOST structs (holding device pointers).
 *  - The library allocates no device memory.  Every scratch byte comes from the
 *    caller's `workspace` (size reported by gnn_plan_query / the *_workspace_bytes
 *    helpers; must be 256-byte aligned).  Every call that takes a `cache` or a
 *    `workspace` also takes its size in bytes and returns GNN_ERR_BUFFER_TOO_SMALL,
 *    before any launch, when that is below what gnn_plan_query reported for the plan.
 *  - Every call only enqueues kernels on `hip_stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and returns; there is no host
 *    synchronisation unless the entry point says otherwise.
 *  - All argument checks run before the first launch, so a call that returns
 *    an error has had no side effect.  No entry point aborts or throws.
 *  - Dense tensors are row-major fp32.  Index arrays are int32.  Outputs are
 *    overwritten, not accumulated into, unless an entry point's flag asks for it.
 *  - Sparse matrices are square n x n in CSR (App. D.1, 0-based): rowptr[0] = 0,
 *    rowptr[n] = nnz, column indices strictly ascending inside a row.  Row i is
 *    the aggregating node, col[e] the neighbour whose features it reads.
 */
#ifndef GNN_H
#define GNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GNN_OK = 0,
    GNN_ERR_INVALID_ARG = 1,      /* NULL where a pointer is required, negative size, bad enum, misalignment */
    GNN_ERR_BAD_GRAPH = 2,        /* graph struct inconsistent with the plan (n / nnz mismatch, missing arrays) */
    GNN_ERR_BUFFER_TOO_SMALL = 3, /* a caller buffer is smaller than the size the library reported */
    GNN_ERR_STATE = 4,            /* backward asked to read a cache that no forward has filled */
    GNN_ERR_UNSUPPORTED = 5,      /* shape outside what the kernels handle */
    GNN_ERR_HIP = 6               /* a HIP call or launch failed */
} gnn_status_t;

typedef enum { GNN_LAYER_GCN = 0, GNN_LAYER_GAT = 1, GNN_LAYER_SAGE = 2 } gnn_layer_t;

/* How an AUTO order / backward scheme is chosen for GCN. */
typedef enum {
    GNN_SELECT_PAPER_RULE = 0,    /* the usage conditions of the tables of Sec. 3.1: SpMM cost is taken
                                     to be proportional to the dense width                              */
    GNN_SELECT_CALIBRATED = 1     /* same candidates, compared by gnn_spmm_time_model_us: the time of this
                                     library's SpMM on an MI355X, which is flat below ~32 columns and has a
                                     fixed launch cost (Sec. 4.1 reports that the proportional rule misses
                                     the best scheme where the two widths are close)                    */
} gnn_select_t;

/* Order of the two products of X' = A' X Theta (Sec. 3.1, Table "GCN schemes"). */
typedef enum {
    GNN_ORDER_AUTO = 0,
    GNN_ORDER_TRANSFORM_FIRST = 1, /* A' (X Theta): GEMM, then SpMM of width F_out */
    GNN_ORDER_PROPAGATE_FIRST = 2  /* (A' X) Theta: SpMM of width F_in, then GEMM  */
} gnn_order_t;

/* Backward scheme (Sec. 3.1, Table "GCN schemes"). */
typedef enum {
    GNN_BWD_AUTO = 0,
    GNN_BWD_FUSED_PROPAGATE = 1,  /* H = A'^T G once (width F_out); dTheta = X^T H; dX = H Theta^T       */
    GNN_BWD_SPLIT_PROPAGATE = 2   /* dTheta = (A'X)^T G; dX = A'^T (G Theta^T): SpMMs of width F_in       */
} gnn_bwd_t;

/* What forward keeps for backward (Sec. 3.1 "Caching intermediate values"; Table "GAT caching"). */
typedef enum {
    GNN_CACHE_AUTO = 0,
    GNN_CACHE_NONE = 1,
    GNN_CACHE_AX = 2,                /* GCN: P = A' X                                                    */
    GNN_CACHE_GAT_FEAT = 3,          /* GAT: M = X Theta                                  (4nhk bytes)   */
    GNN_CACHE_GAT_FEAT_NODEATT = 4,  /* GAT: M, s, d                                      (4nh(k+2))     */
    GNN_CACHE_GAT_FEAT_EDGE = 5      /* GAT: M, edge weights alpha, LeakyReLU mask        (4nhk + 5qh)   */
} gnn_cache_t;

/*
 * A graph: host struct of device arrays.
 *   csr_*      the matrix by rows (always required).  csr_val may be NULL for GAT
 *              (attention ignores edge weights, Sec. 3.2) - never for GCN.
 *   csr_erow   optional for GCN, required for GAT: row index of every stored entry (erow[e] = i for
 *              rowptr[i] <= e < rowptr[i+1]), as written by gnn_expand_ptr.  With it
 *              the sparse kernels split work by equal numbers of entries, which
 *              keeps hub rows from serialising; without it they fall back to one
 *              lane group per row (same results, slower on skewed graphs).
 *   csc_*      the same matrix by columns, i.e. the CSR arrays of its transpose:
 *              colptr[n+1], row[nnz] ascending inside a column, perm[nnz] mapping a
 *              CSC slot to the CSR slot of the same entry, val = csr_val[perm]
 *              (may be NULL: then values are fetched through perm), ecol = the
 *              expanded column index per CSC slot (like csr_erow: optional for GCN,
 *              required by gat_layer_bwd).
 *              Needed by every backward pass unless `symmetric` is set.
 *   symmetric  nonzero promises A'^T == A' (pattern and values); the CSC arrays
 *              are then ignored and may be NULL.  Only meaningful for GCN and SAGE.
 */
typedef struct {
    int32_t n, nnz;
    const int32_t *csr_rowptr, *csr_col;
    const float *csr_val;
    const int32_t *csr_erow;
    const int32_t *csc_colptr, *csc_row, *csc_perm;
    const float *csc_val;
    const int32_t *csc_ecol;
    int32_t symmetric;
} gnn_graph_t;

typedef struct {
    gnn_layer_t layer;
    int32_t n, nnz;           /* nodes, stored entries (self-loops included)                    */
    int32_t f_in;             /* m                                                              */
    int32_t f_out;            /* k, per head for GAT                                            */
    int32_t heads;            /* GAT only (GCN, SAGE: 1)                                        */
    int32_t need_input_grad;  /* 0: backward skips dX (first layer of a network)                */
    int32_t has_bias;         /* forward adds b, backward writes db                             */
    int32_t fuse_relu;        /* GCN, SAGE: forward applies ReLU, backward masks dY by [Y > 0]  */
    float leaky_slope;        /* GAT only: beta of LeakyReLU                                    */
    gnn_order_t order;        /* AUTO or a forced choice                                        */
    gnn_bwd_t bwd;
    gnn_cache_t cache;
    gnn_select_t selection;   /* how AUTO decides (GCN, SAGE: order and scheme; GAT: the cache variant) */
    int32_t constant_input;   /* GCN, SAGE with the A'X cache: the caller promises that X and the graph
                                 are the same in every forward call until gnn_plan_reset_cache
                                 (a first layer whose input features never change).  Forward then
                                 computes A'X only while the cache is empty, and AUTO counts that
                                 SpMM as free.  A GCN layer reads X only in that first call.       */
    int32_t fuse_elu;         /* GAT only: forward applies ELU (alpha = 1) after the bias, backward
                                 multiplies dY by its derivative taken from the output Y            */
} gnn_plan_desc_t;

typedef struct {
    gnn_order_t order;        /* resolved, never AUTO */
    gnn_bwd_t bwd;
    gnn_cache_t cache;
    size_t cache_bytes;       /* size of the `cache` buffer fwd writes and bwd reads            */
    size_t workspace_bytes;   /* max over fwd and bwd                                           */
    int64_t transient_fwd;    /* number of fp32 transients of the paper's tables (nk / nm ...)  */
    int64_t transient_bwd;
    int64_t spmm_width_fwd;   /* summed dense widths of the SpMMs the scheme runs               */
    int64_t spmm_width_bwd;
} gnn_plan_info_t;

typedef struct gnn_plan gnn_plan_t;

/*
 * gnn_plan_create - choose ordering, backward scheme and cache policy (host only, no device work).
 *
 * GCN, caching allowed (cache = AUTO or AX)        [Table "GCN schemes with caching"]:
 *     with dX:  F_out <  F_in    -> transform-first + fused-propagate, no cache
 *               F_out >= F_in    -> propagate-first caching A'X + split-propagate reading it
 *     no dX:    F_out <  F_in/2  -> transform-first + fused-propagate
 *               F_out >= F_in/2  -> propagate-first with cache + split-propagate with cache
 * GCN, caching forbidden (cache = NONE)            [Table "GCN schemes"]:
 *     forward:  F_out < F_in -> transform-first, else propagate-first
 *     backward: with dX: F_out < 2 F_in -> fused-propagate, else split-propagate
 *               no dX:   F_out <   F_in -> fused-propagate, else split-propagate
 * With selection = CALIBRATED the same candidate schemes are compared by the summed model time
 * of their SpMMs instead (the GEMMs are the same in every scheme); ties go to the rule's choice.
 * With constant_input (and caching allowed) the forward SpMM of the cached scheme costs nothing.
 * Forced `order` / `bwd` values override the rule; cache = AX needs order = PROPAGATE_FIRST
 * (else GNN_ERR_INVALID_ARG).  GAT: order is fixed (node-attention form, App. B);
 * cache AUTO -> GNN_CACHE_GAT_FEAT_EDGE, the fastest variant of Sec. 4.2; with selection = CALIBRATED ->
 * GNN_CACHE_GAT_FEAT_NODEATT, the fastest measured on an MI355X (the edge passes rebuild alpha from four
 * floats per node for less than reading five bytes per entry and head costs).
 * The plan is a host object owned by the caller until gnn_plan_destroy.
 */
gnn_status_t gnn_plan_create(const gnn_plan_desc_t *desc, gnn_plan_t **out);
gnn_status_t gnn_plan_query(const gnn_plan_t *plan, gnn_plan_info_t *out);
void gnn_plan_destroy(gnn_plan_t *plan);

/* Forget that a forward pass has filled the cache (constant_input: the next forward recomputes A'X). */
gnn_status_t gnn_plan_reset_cache(gnn_plan_t *plan);

/*
 * gnn_spmm_time_model_us - the time model behind GNN_SELECT_CALIBRATED (host only): microseconds of
 * one SpMM of dense width f on a graph of n nodes and nnz entries with this library's kernels on an
 * MI355X:  t = 12 + nnz * max(13, c * f) * 1e-6,  c = 0.32 ps per entry and column while the dense
 * operand (D = 4 n f bytes) is below 70 MB, else 0.32 + 0.045 log2(D / 70 MB), at most 0.53.
 * Fitted to measurements on R-MAT graphs of 2^11 .. 2^22 nodes; within about 20 % of them.
 */
double gnn_spmm_time_model_us(int64_t n, int64_t nnz, int32_t f);

/*
 * gcn_layer_fwd - Y = A' X W + 1 b^T (Eq. gcn-fwd), optionally ReLU.
 *   X [n, f_in], W [f_in, f_out], b [f_out] or NULL, Y [n, f_out]           (device)
 *   cache      cache_bytes >= the plan's; written when the plan caches A'X, may be NULL (size 0) otherwise
 *   workspace  workspace_bytes >= the plan's
 * Errors: INVALID_ARG (NULL X / W / Y, b missing while has_bias), BAD_GRAPH
 * (n / nnz differ from the plan, csr arrays or csr_val NULL), BUFFER_TOO_SMALL (cache or
 * workspace smaller than gnn_plan_query reports).
 */
gnn_status_t gcn_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *b, float *Y, void *cache, size_t cache_bytes,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * gcn_layer_bwd - dW = X^T A'^T dY, db = dY^T 1, dX = A'^T dY W^T (Eqs. gcn-bwd-*).
 *   X   [n, f_in]; may be NULL when the plan caches A'X (App. A: the input is then not needed)
 *   Y   [n, f_out] forward output; required iff fuse_relu (its sign gives the ReLU mask)
 *   dY  [n, f_out]; dW [f_in, f_out]; db [f_out] (required iff has_bias);
 *   dX  [n, f_in]  (required iff need_input_grad, ignored otherwise)
 * Errors: as forward, plus STATE when the plan caches A'X and no forward has run
 * on this plan since creation, BAD_GRAPH when the graph is not symmetric and
 * the CSC arrays are missing.
 */
gnn_status_t gcn_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *Y, const float *dY, float *dW, float *db, float *dX,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/*
 * sage_layer_fwd / sage_layer_bwd - a GraphSAGE layer, the other layer that Sec. 3.1 "Generalizability"
 * names for the same chained product:  Y = X W_self + A' X W_neigh + 1 b^T  (optionally ReLU), with A'
 * the row-normalised pattern (gnn_aggregator_weights, GNN_AGG_MEAN) or any other entry values.
 * The plan is made with layer = GNN_LAYER_SAGE; order, backward scheme, cache (A'X) and their AUTO
 * choice are those of GCN, since the SpMM widths are the same (F_out transform-first, F_in propagate-first).
 *   X [n, f_in], W_self / W_neigh [f_in, f_out], b [f_out] or NULL, Y [n, f_out]
 *   backward: dW_self = X^T G, dW_neigh = (A'X)^T G, db = G^T 1, dX = G W_self^T + A'^T G W_neigh^T
 *   (G = dY, masked by [Y > 0] with fuse_relu).  X is needed by backward in every scheme.
 * cache / workspace sizes: gnn_plan_query.  Errors as gcn_layer_fwd / gcn_layer_bwd.
 */
gnn_status_t sage_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W_self,
                            const float *W_neigh, const float *b, float *Y, void *cache, size_t cache_bytes,
                            void *workspace, size_t workspace_bytes, void *hip_stream);
gnn_status_t sage_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W_self,
                            const float *W_neigh, const float *Y, const float *dY, float *dW_self,
                            float *dW_neigh, float *db, float *dX, void *cache, size_t cache_bytes,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * gat_layer_fwd - multi-head GAT forward (Eqs. gat-fwd, gat-fwd-att), heads concatenated.
 *   X [n, f_in], W [f_in, heads*f_out], a_src / a_dst [heads, f_out], b [heads*f_out] or NULL,
 *   Y [n, heads*f_out] laid out [n][head][f_out] (head is the middle axis, Sec. 3.2);
 *   with fuse_elu, Y = ELU(aggregate + b) (the activation of the paper's two-layer GAT, Sec. 4).
 *   a_src multiplies the features of the row (aggregating) node, a_dst those of
 *   the column (neighbour) node: logit(i, j) = <a_src, m_i> + <a_dst, m_j>.
 *   The softmax runs over the stored entries of row i; csr_val is ignored.
 *   cache layout (all fp32 unless noted, each block 256-byte aligned, in this order):
 *     GAT_FEAT:         M [n][h][k]
 *     GAT_FEAT_NODEATT: M, s [n][h], d [n][h]
 *     GAT_FEAT_EDGE:    M, alpha [nnz][h], mask [nnz][h] uint8 (1 where the logit is > 0)
 */
gnn_status_t gat_layer_fwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *a_src, const float *a_dst, const float *b, float *Y,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/*
 * gat_layer_bwd - gradients of Sec. "GAT Backward Pass": dW [f_in, h*k], da_src / da_dst [h, k],
 *   db [h*k] (iff has_bias), dX [n, f_in] (iff need_input_grad).  Needs the CSC arrays and perm.
 *   Y [n, h*k]: the forward output; required iff fuse_elu (ELU'(x) = 1 for x > 0, else Y + 1).
 *   Whatever the cache variant did not keep is recomputed with the forward kernels.
 */
gnn_status_t gat_layer_bwd(gnn_plan_t *plan, const gnn_graph_t *graph, const float *X, const float *W,
                           const float *a_src, const float *a_dst, const float *Y, const float *dY,
                           float *dW, float *da_src, float *da_dst, float *db, float *dX,
                           void *cache, size_t cache_bytes, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/* ---- preprocessing: integer kernels and the normalisation (Sec. "GCN Forward Pass") ---- */

/*
 * gnn_add_self_loops_degree - pattern of A + I and its row degrees.
 *   in:  rowptr [n+1], col [nnz] (ascending rows; a diagonal entry may already be there)
 *   out: rowptr_out [n+1], col_out [capacity nnz + n], deg_out [n] = entries per row of A + I
 *   nnz_out_host: HOST pointer; receives rowptr_out[n].  This call synchronises the stream.
 *   workspace: gnn_scan_workspace_bytes(n) bytes.
 */
gnn_status_t gnn_add_self_loops_degree(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col,
                                       int32_t *rowptr_out, int32_t *col_out, int32_t *deg_out,
                                       int32_t *nnz_out_host, void *workspace, size_t workspace_bytes,
                                       void *hip_stream);
size_t gnn_scan_workspace_bytes(int32_t n);

/* val_out[e] = 1 / sqrt(deg[i] * deg[col[e]]) for every stored entry e of row i. */
gnn_status_t gnn_gcn_normalize(int32_t n, const int32_t *rowptr, const int32_t *col, const int32_t *deg,
                               float *val_out, void *hip_stream);

/*
 * gnn_aggregator_weights - entry values for the other layers with the same chained product A' X Theta
 * (Sec. 3.1 "Generalizability"; App. "GCN Forward Pass": mean aggregation is D A X Theta), on the
 * pattern of A + I with the degrees written by gnn_add_self_loops_degree:
 *   GNN_AGG_GCN_SYM  1 / sqrt(deg_i deg_j)            (what gnn_gcn_normalize writes)
 *   GNN_AGG_MEAN     1 / deg_i                         (row-normalised: mean over N(i) and i itself)
 *   GNN_AGG_GIN_SUM  1, and 1 + eps on the diagonal    (the sum aggregation of a GIN layer)
 * The mean weights are not symmetric: the graph then needs its CSC arrays (symmetric = 0) for backward.
 */
typedef enum { GNN_AGG_GCN_SYM = 0, GNN_AGG_MEAN = 1, GNN_AGG_GIN_SUM = 2 } gnn_aggregator_t;
gnn_status_t gnn_aggregator_weights(gnn_aggregator_t kind, float eps, int32_t n, const int32_t *rowptr,
                                    const int32_t *col, const int32_t *deg, float *val_out, void *hip_stream);

/*
 * gnn_csr_transpose - CSC arrays of a CSR matrix (App. D.1): colptr_out [n+1], row_out [nnz]
 * ascending inside every column, perm_out [nnz] (CSC slot -> CSR slot).  Deterministic:
 * a stable radix sort of the row-major entries by column.
 */
gnn_status_t gnn_csr_transpose(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col,
                               int32_t *colptr_out, int32_t *row_out, int32_t *perm_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream);
size_t gnn_transpose_workspace_bytes(int32_t n, int32_t nnz);

/* out[e] = i for ptr[i] <= e < ptr[i+1]  (the COO row array of App. D.2, from CSR). */
gnn_status_t gnn_expand_ptr(int32_t n, int32_t nnz, const int32_t *ptr, int32_t *out, void *hip_stream);

/* out[p] = in[perm[p]] (e.g. csc_val from csr_val). */
gnn_status_t gnn_gather_f32(int64_t count, const float *in, const int32_t *perm, float *out, void *hip_stream);

/* ---- the sparse and dense operators on their own (App. E) ---- */

/*
 * gnn_spmm_csr - C = A B (App. E.1).  B, C [n, f].  val NULL = all ones.
 *   erow: optional expanded row index (see gnn_graph_t); selects the entry-balanced kernel.
 *   bias [f] or NULL, relu (0 or 1; anything else is GNN_ERR_INVALID_ARG): fused epilogue C = relu(A B + 1 b^T).
 *   workspace: gnn_spmm_workspace_bytes(n, nnz, f) bytes (only used with erow): partial rows of the
 *   blocks and, when f is not a multiple of 4, a copy of B with rows padded to the next multiple of 4.
 *   B and C may start at any 4-byte aligned address; 16-byte aligned rows take the fastest kernel.
 */
gnn_status_t gnn_spmm_csr(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col, const float *val,
                          const int32_t *erow, const float *B, int32_t f, float *C,
                          const float *bias, int32_t relu,
                          void *workspace, size_t workspace_bytes, void *hip_stream);
size_t gnn_spmm_workspace_bytes(int32_t n, int32_t nnz, int32_t f);

/*
 * gnn_spmm_csr_static - gnn_spmm_csr for callers that cannot allocate device memory and have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as gnn_spmm_csr; the scratch (partial rows, padded operand) is a device
 * array of GNN_STATIC_SCRATCH_BYTES bytes inside the library, one copy per GPU, held until the process ends.
 * The call allocates nothing and frees nothing.
 *   Errors: as gnn_spmm_csr; GNN_ERR_BUFFER_TOO_SMALL when gnn_spmm_workspace_bytes(n, nnz, f) exceeds
 *   GNN_STATIC_SCRATCH_BYTES (then use gnn_spmm_csr with a workspace of that size).
 *   The first call on a device looks up the array's address there (make it outside a graph capture).
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 *   streams, or several host threads) race; calls on one stream are ordered and safe.  Nothing in the
 *   array needs clearing between calls: every partial row is written before it is read.
 */
#define GNN_STATIC_SCRATCH_BYTES (32u << 20)
gnn_status_t gnn_spmm_csr_static(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col, const float *val,
                                 const int32_t *erow, const float *B, int32_t f, float *C,
                                 const float *bias, int32_t relu, void *hip_stream);

/*
 * Storage formats other than CSR (App. D.2 coordinate, D.3 ELLPACK, D.4 hybrid) and SpMM on them, for the
 * format comparison of App. E.1.  The layers never use them.
 *   ELLPACK arrays ell_col / ell_val [t][n] are slot-major: slot j of row i at [j * n + i]; a row's stored
 *   entries fill its slots from the front, padding has column -1 and value 0.  With t >= the longest row this
 *   is plain ELLPACK (p = t); with a smaller t it is the hybrid format: the first t entries of every row in
 *   the ELLPACK arrays, the others row-major in coordinate arrays coo_row / coo_col / coo_val [rest_nnz].
 *
 * gnn_csr_hyb_count - rest_ptr_out [n+1] (device) = exclusive scan of max(0, row length - t);
 *   rest_nnz_out_host / max_row_out_host: HOST pointers receiving rest_ptr_out[n] and the longest row
 *   (either may be NULL).  Synchronises the stream.  workspace: gnn_hyb_workspace_bytes(n).
 * gnn_csr_to_hyb - fills the arrays; val NULL = all ones.  rest_ptr NULL: no coordinate part is written
 *   (entries beyond slot t are dropped, so pass t >= the longest row).  t = 0: everything goes to the
 *   coordinate arrays (ell_* may be NULL).
 * gnn_spmm_ell - C = A B from the ELLPACK arrays.  Deterministic.
 * gnn_spmm_coo - C = A B (accumulate = 0: C is cleared first) or C += A B (accumulate != 0) from
 *   coordinate arrays in any order; val NULL = all ones.  Uses fp32 atomic additions: the result is
 *   reproducible only up to fp32 rounding.
 * gnn_spmm_hyb - gnn_spmm_ell on the first t slots, then gnn_spmm_coo accumulating the rest.
 *   B, C [n, f] row-major.  Errors: GNN_ERR_INVALID_ARG for negative sizes / NULL required pointers.
 */
size_t gnn_hyb_workspace_bytes(int32_t n);
gnn_status_t gnn_csr_hyb_count(int32_t n, const int32_t *rowptr, int32_t t, int32_t *rest_ptr_out,
                               int32_t *rest_nnz_out_host, int32_t *max_row_out_host,
                               void *workspace, size_t workspace_bytes, void *hip_stream);
gnn_status_t gnn_csr_to_hyb(int32_t n, int32_t t, const int32_t *rowptr, const int32_t *col, const float *val,
                            const int32_t *rest_ptr, int32_t *ell_col, float *ell_val,
                            int32_t *coo_row, int32_t *coo_col, float *coo_val, void *hip_stream);
gnn_status_t gnn_spmm_ell(int32_t n, int32_t t, const int32_t *ell_col, const float *ell_val,
                          const float *B, int32_t f, float *C, void *hip_stream);
gnn_status_t gnn_spmm_coo(int32_t n, int64_t nnz, const int32_t *row, const int32_t *col, const float *val,
                          const float *B, int32_t f, float *C, int32_t accumulate, void *hip_stream);
gnn_status_t gnn_spmm_hyb(int32_t n, int32_t t, const int32_t *ell_col, const float *ell_val,
                          int64_t rest_nnz, const int32_t *coo_row, const int32_t *coo_col, const float *coo_val,
                          const float *B, int32_t f, float *C, void *hip_stream);

/*
 * gnn_sddmm_csr - D_e = val_e * <B_i, Ct_j> for every stored entry e = (i, j) (App. E.2),
 *   batched over `heads` with the head as the middle axis: B, Ct [n][heads][f], D [nnz][heads].
 *   Ct is the transpose of the paper's C (row j = column j of C).  val NULL = all ones.
 *   erow [nnz]: the row i of every entry (gnn_expand_ptr of the row pointers); the kernel is
 *   one thread per (entry, head), so it needs no row pointers.
 */
gnn_status_t gnn_sddmm_csr(int32_t n, int32_t nnz, const int32_t *erow, const int32_t *col, const float *val,
                           const float *B, const float *Ct, int32_t heads, int32_t f, float *D,
                           void *hip_stream);

/*
 * gnn_gat_aggregate_csr - the edge phase of the GAT forward pass as one operator (Eqs. gat-fwd-att, gat-fwd):
 *   alpha_e = softmax over the stored entries of row i of LeakyReLU(s_i + d_j)   per head,
 *   Y_{i,p,:} = sum_e alpha_{e,p} M_{col e,p,:} (+ bias, then ELU if elu != 0),
 * in a single pass over the entries: the logits, the running softmax and the weighted sum stay in registers,
 * no per-edge array is written.  M, Y [n][heads][f]; s, d [n][heads] (App. B: s_i = <a_src, m_i>,
 * d_j = <a_dst, m_j>); bias [heads * f] or NULL;
 * stat_out [n][heads][2] receives (row maximum of the LeakyReLU'd logits, sum of exp(. - maximum)), from which
 * alpha_e = exp(w_e - max) / sum.  erow [nnz]: row of every entry (gnn_expand_ptr).
 *   f: a multiple of 4 with f / 4 a power of two, at most 256; M, Y and bias 16-byte aligned; n below 2^24,
 *   M below 4 GiB and nnz * heads below 2^30 (the gathers use 32-bit byte offsets)
 *   (GNN_ERR_UNSUPPORTED otherwise: gat_layer_fwd then runs the steps as separate kernels).
 *   workspace: gnn_gat_aggregate_workspace_bytes(nnz, heads, f).
 */
gnn_status_t gnn_gat_aggregate_csr(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *erow,
                                   const int32_t *col, const float *M, const float *s, const float *d,
                                   int32_t heads, int32_t f, float leaky_slope, const float *bias, int32_t elu,
                                   float *Y, float *stat_out, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);
size_t gnn_gat_aggregate_workspace_bytes(int32_t nnz, int32_t heads, int32_t f);

/*
 * gnn_gemm - C = op(A) op(B) on the matrix cores: fp32 operands and results; fp32 accumulation,
 *   except that the transposed-A form accumulates in fp64 (its reduction runs over all nodes).
 *   trans_a == 0: A is [M, K] else A is [K, M] and used transposed (then K may be huge:
 *   the product is split along K and reduced in a fixed order; deterministic).
 *   trans_b == 0: B is [K, N] else B is [N, K].  C is [M, N].  All row-major, dense (ld = columns).
 *   bias [N] or NULL, relu: fused epilogue.  Supported: (0,0), (0,1), (1,0).
 *   relu is a flag word: GNN_GEMM_RELU (1) applies max(., 0); GNN_GEMM_ACCUMULATE (4) adds the
 *   product (and bias) to what C holds before the ReLU, trans_a == 0 only (GNN_ERR_UNSUPPORTED
 *   otherwise); any other bit is GNN_ERR_INVALID_ARG.
 *   workspace: gnn_gemm_workspace_bytes(trans_a, trans_b, M, N, K); required for (0,0) (holds B^T)
 *   and (1,0) (holds the partial products); (0,1) needs none.
 */
enum { GNN_GEMM_RELU = 1, GNN_GEMM_ACCUMULATE = 4 };
gnn_status_t gnn_gemm(int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K,
                      const float *A, const float *B, float *C, const float *bias, int32_t relu,
                      void *workspace, size_t workspace_bytes, void *hip_stream);
size_t gnn_gemm_workspace_bytes(int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K);

/*
 * gnn_softmax_xent - sum-reduced softmax cross-entropy over the rows of Z [n, c] with
 * integer labels [n]; writes dZ = softmax(Z) - onehot [n, c] and loss_out[0] (device, fp32).
 * (The loss used on the two-layer GCN workload; not part of a layer.)
 *   workspace: 4 * ceil(n / 256) bytes.
 */
gnn_status_t gnn_softmax_xent(int32_t n, int32_t c, const float *Z, const int32_t *labels, float *dZ,
                              float *loss_out, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * gnn_sum_squared_error - loss_out[0] = 1/2 sum (Z - T)^2 over `count` elements and dZ = Z - T
 * (the squared-error loss of the paper's full-network runs, Sec. 4, sum-reduced so that the
 * gradient entries are O(1)).  Deterministic two-stage sum.  workspace: 4096 bytes.
 */
gnn_status_t gnn_sum_squared_error(int64_t count, const float *Z, const float *T, float *dZ, float *loss_out,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

const char *gnn_status_string(gnn_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* GNN_H */
