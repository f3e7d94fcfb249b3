/*
 * A caller of the C ABI written in C: no Python, no torch.  It builds a small ring-with-chords graph on the
 * host, runs the preprocessing entry points, one GCN layer forward and backward (adaptive plan), and
 * checks every output against a dense double-precision evaluation of the layer's definition
 * (A' = D^-1/2 (A + I) D^-1/2, Y = A' X W + b; dW = X^T A'^T G, db = G^T 1, dX = A'^T G W^T).
 * Prints "ok" and returns 0 when all entries agree within 1e-4 (1 + |ref|).
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include "gnn.h"

#define N 96
#define M 20
#define K 12

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define GNN_CHECK(x) do { gnn_status_t s_ = (x); if (s_ != GNN_OK) { fprintf(stderr, "%s at line %d\n", gnn_status_string(s_), __LINE__); return 3; } } while (0)

static void *dev_copy(const void *host, size_t bytes) {
    void *p = NULL;
    if (hipMalloc(&p, bytes ? bytes : 4) != hipSuccess) return NULL;
    if (host && bytes && hipMemcpy(p, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return p;
}

static float pseudo(unsigned *state) {              /* small LCG, values in [-1, 1) */
    *state = *state * 1664525u + 1013904223u;
    return (float)((*state >> 8) & 0xFFFF) / 32768.0f - 1.0f;
}

static int compare(const char *name, const float *got, const double *ref, int count) {
    for (int i = 0; i < count; ++i)
        if (!(fabs((double)got[i] - ref[i]) <= 1e-4 * (1.0 + fabs(ref[i])))) {
            fprintf(stderr, "%s[%d]: got %.7g, expected %.7g\n", name, i, got[i], ref[i]);
            return 1;
        }
    return 0;
}

int main(void) {
    /* undirected pattern without diagonal: i ~ i+1, i ~ i+7 (mod N), columns ascending */
    static int adj[N][N];
    for (int i = 0; i < N; ++i) {
        const int nb[2] = {(i + 1) % N, (i + 7) % N};
        for (int t = 0; t < 2; ++t) { adj[i][nb[t]] = 1; adj[nb[t]][i] = 1; }
    }
    int32_t rowptr[N + 1], col[N * 4];
    int nnz = 0;
    for (int i = 0; i < N; ++i) {
        rowptr[i] = nnz;
        for (int j = 0; j < N; ++j) if (adj[i][j]) col[nnz++] = j;
    }
    rowptr[N] = nnz;

    static float X[N * M], W[M * K], b[K], G[N * K];
    unsigned st = 12345u;
    for (int i = 0; i < N * M; ++i) X[i] = pseudo(&st);
    for (int i = 0; i < M * K; ++i) W[i] = 0.3f * pseudo(&st);
    for (int i = 0; i < K; ++i) b[i] = pseudo(&st);
    for (int i = 0; i < N * K; ++i) G[i] = pseudo(&st);

    /* ---- device side: preprocessing ---- */
    int32_t *d_rp = dev_copy(rowptr, sizeof rowptr), *d_col = dev_copy(col, sizeof(int32_t) * nnz);
    int32_t *d_rp2 = dev_copy(NULL, sizeof(int32_t) * (N + 1)), *d_col2 = dev_copy(NULL, sizeof(int32_t) * (nnz + N));
    int32_t *d_deg = dev_copy(NULL, sizeof(int32_t) * N);
    void *scan_ws = dev_copy(NULL, gnn_scan_workspace_bytes(N));
    if (!d_rp || !d_col || !d_rp2 || !d_col2 || !d_deg || !scan_ws) { fprintf(stderr, "device allocation failed\n"); return 2; }
    int32_t q = 0;
    GNN_CHECK(gnn_add_self_loops_degree(N, nnz, d_rp, d_col, d_rp2, d_col2, d_deg, &q, scan_ws,
                                        gnn_scan_workspace_bytes(N), NULL));
    if (q != nnz + N) { fprintf(stderr, "self-loops: %d entries, expected %d\n", q, nnz + N); return 1; }
    float *d_val = dev_copy(NULL, sizeof(float) * q);
    int32_t *d_erow = dev_copy(NULL, sizeof(int32_t) * q);
    if (!d_val || !d_erow) { fprintf(stderr, "device allocation failed\n"); return 2; }
    GNN_CHECK(gnn_gcn_normalize(N, d_rp2, d_col2, d_deg, d_val, NULL));
    GNN_CHECK(gnn_expand_ptr(N, q, d_rp2, d_erow, NULL));

    gnn_graph_t graph;
    memset(&graph, 0, sizeof graph);
    graph.n = N; graph.nnz = q;
    graph.csr_rowptr = d_rp2; graph.csr_col = d_col2; graph.csr_val = d_val; graph.csr_erow = d_erow;
    graph.symmetric = 1;                                  /* A' equals its transpose: no CSC arrays needed */

    /* ---- plan, buffers, one forward and one backward ---- */
    gnn_plan_desc_t desc;
    memset(&desc, 0, sizeof desc);
    desc.layer = GNN_LAYER_GCN; desc.n = N; desc.nnz = q; desc.f_in = M; desc.f_out = K; desc.heads = 1;
    desc.need_input_grad = 1; desc.has_bias = 1;
    desc.order = GNN_ORDER_AUTO; desc.bwd = GNN_BWD_AUTO; desc.cache = GNN_CACHE_AUTO;
    gnn_plan_t *plan = NULL;
    gnn_plan_info_t info;
    GNN_CHECK(gnn_plan_create(&desc, &plan));
    GNN_CHECK(gnn_plan_query(plan, &info));
    void *ws = dev_copy(NULL, info.workspace_bytes), *cache = info.cache_bytes ? dev_copy(NULL, info.cache_bytes) : NULL;
    float *d_X = dev_copy(X, sizeof X), *d_W = dev_copy(W, sizeof W), *d_b = dev_copy(b, sizeof b), *d_G = dev_copy(G, sizeof G);
    float *d_Y = dev_copy(NULL, sizeof(float) * N * K), *d_dW = dev_copy(NULL, sizeof W), *d_db = dev_copy(NULL, sizeof b);
    float *d_dX = dev_copy(NULL, sizeof X);
    if (!ws || !d_X || !d_W || !d_b || !d_G || !d_Y || !d_dW || !d_db || !d_dX) { fprintf(stderr, "device allocation failed\n"); return 2; }
    GNN_CHECK(gcn_layer_fwd(plan, &graph, d_X, d_W, d_b, d_Y, cache, info.cache_bytes, ws, info.workspace_bytes, NULL));
    GNN_CHECK(gcn_layer_bwd(plan, &graph, d_X, d_W, NULL, d_G, d_dW, d_db, d_dX, cache, info.cache_bytes, ws,
                            info.workspace_bytes, NULL));
    HIP_OK(hipDeviceSynchronize());
    static float Y[N * K], dW[M * K], db[K], dX[N * M];
    HIP_OK(hipMemcpy(Y, d_Y, sizeof Y, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dW, d_dW, sizeof dW, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(db, d_db, sizeof db, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dX, d_dX, sizeof dX, hipMemcpyDeviceToHost));

    /* ---- the definition, dense and in double ---- */
    static double A[N][N], AX[N][M], rY[N * K], AG[N][K], rdW[M * K], rdb[K], rdX[N * M];
    int deg[N];
    for (int i = 0; i < N; ++i) { deg[i] = 1; for (int j = 0; j < N; ++j) deg[i] += adj[i][j]; }
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j)
            A[i][j] = (adj[i][j] || i == j) ? 1.0 / sqrt((double)deg[i] * deg[j]) : 0.0;
    for (int i = 0; i < N; ++i)
        for (int c = 0; c < M; ++c) { double s = 0; for (int j = 0; j < N; ++j) s += A[i][j] * X[j * M + c]; AX[i][c] = s; }
    for (int i = 0; i < N; ++i)
        for (int o = 0; o < K; ++o) { double s = b[o]; for (int c = 0; c < M; ++c) s += AX[i][c] * W[c * K + o]; rY[i * K + o] = s; }
    for (int i = 0; i < N; ++i)                       /* A'^T G (A' is symmetric) */
        for (int o = 0; o < K; ++o) { double s = 0; for (int j = 0; j < N; ++j) s += A[j][i] * G[j * K + o]; AG[i][o] = s; }
    for (int c = 0; c < M; ++c)
        for (int o = 0; o < K; ++o) { double s = 0; for (int i = 0; i < N; ++i) s += X[i * M + c] * AG[i][o]; rdW[c * K + o] = s; }
    for (int o = 0; o < K; ++o) { double s = 0; for (int i = 0; i < N; ++i) s += G[i * K + o]; rdb[o] = s; }
    for (int i = 0; i < N; ++i)
        for (int c = 0; c < M; ++c) { double s = 0; for (int o = 0; o < K; ++o) s += AG[i][o] * W[c * K + o]; rdX[i * M + c] = s; }

    int bad = compare("Y", Y, rY, N * K) | compare("dW", dW, rdW, M * K) | compare("db", db, rdb, K) |
              compare("dX", dX, rdX, N * M);
    gnn_plan_destroy(plan);
    if (bad) return 1;
    printf("ok: GCN layer from C, n=%d nnz=%d %d->%d, order=%d bwd=%d cache=%d\n", N, (int)q, M, K, (int)info.order,
           (int)info.bwd, (int)info.cache);
    return 0;
}
