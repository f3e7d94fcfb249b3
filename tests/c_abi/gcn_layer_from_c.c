/*
 * A caller of the C ABI written in C: no Python, no torch.  It builds a small ring-with-chords graph on the
 * host, runs the preprocessing entry points, one GCN layer forward and backward (adaptive plan), and
 * checks every output against a dense double-precision evaluation of the layer's definition
 * (A' = D^-1/2 (A + I) D^-1/2, Y = A' X W + b; dW = X^T A'^T G, db = G^T 1, dX = A'^T G W^T).
 * Then one GAT layer (2 heads, every caching variant) on a directed version of the graph: transpose, expanded
 * indices, forward and backward, against dense loops over the equations of the forward and backward pass
 * (row softmax of LeakyReLU(s_i + d_j) over the stored entries; the chain rule through it).
 * Prints "ok" lines and returns 0 when all entries agree within 1e-4 (1 + |ref|).
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

#define H 2                 /* heads */
#define KH 4                /* features per head */
#define F (H * KH)

/* One GAT layer on the directed graph i <- i+1, i <- i+7, i <- 3i+2 (mod N) plus self-loops. */
static int gat_from_c(void) {
    static int pat[N][N];                                 /* pat[i][j]: row i aggregates from j */
    for (int i = 0; i < N; ++i) { pat[i][(i + 1) % N] = 1; pat[i][(i + 7) % N] = 1; pat[i][(3 * i + 2) % N] = 1; }
    for (int i = 0; i < N; ++i) pat[i][i] = 0;            /* self-loops are added by the library */
    int32_t rowptr[N + 1], col[N * 3];
    int nnz = 0;
    for (int i = 0; i < N; ++i) {
        rowptr[i] = nnz;
        for (int j = 0; j < N; ++j) if (pat[i][j]) col[nnz++] = j;
    }
    rowptr[N] = nnz;
    static float X[N * M], W[M * F], as[F], ad[F], b[F], G[N * F];
    unsigned st = 777u;
    for (int i = 0; i < N * M; ++i) X[i] = pseudo(&st);
    for (int i = 0; i < M * F; ++i) W[i] = 0.4f * pseudo(&st);
    for (int i = 0; i < F; ++i) { as[i] = pseudo(&st); ad[i] = pseudo(&st); b[i] = pseudo(&st); }
    for (int i = 0; i < N * F; ++i) G[i] = pseudo(&st);
    const float beta = 0.2f;

    /* preprocessing on the device: self-loops, transpose, expanded row / column indices */
    int32_t *d_rp = dev_copy(rowptr, sizeof rowptr), *d_col = dev_copy(col, sizeof(int32_t) * nnz);
    int32_t *d_rp2 = dev_copy(NULL, sizeof(int32_t) * (N + 1)), *d_col2 = dev_copy(NULL, sizeof(int32_t) * (nnz + N));
    int32_t *d_deg = dev_copy(NULL, sizeof(int32_t) * N);
    void *scan_ws = dev_copy(NULL, gnn_scan_workspace_bytes(N));
    if (!d_rp || !d_col || !d_rp2 || !d_col2 || !d_deg || !scan_ws) { fprintf(stderr, "device allocation failed\n"); return 2; }
    int32_t q = 0;
    GNN_CHECK(gnn_add_self_loops_degree(N, nnz, d_rp, d_col, d_rp2, d_col2, d_deg, &q, scan_ws,
                                        gnn_scan_workspace_bytes(N), NULL));
    if (q != nnz + N) { fprintf(stderr, "self-loops: %d entries, expected %d\n", q, nnz + N); return 1; }
    int32_t *d_cp = dev_copy(NULL, sizeof(int32_t) * (N + 1)), *d_row = dev_copy(NULL, sizeof(int32_t) * q);
    int32_t *d_perm = dev_copy(NULL, sizeof(int32_t) * q), *d_erow = dev_copy(NULL, sizeof(int32_t) * q);
    int32_t *d_ecol = dev_copy(NULL, sizeof(int32_t) * q);
    const size_t tws = gnn_transpose_workspace_bytes(N, q);
    void *t_ws = dev_copy(NULL, tws);
    if (!d_cp || !d_row || !d_perm || !d_erow || !d_ecol || !t_ws) { fprintf(stderr, "device allocation failed\n"); return 2; }
    GNN_CHECK(gnn_csr_transpose(N, q, d_rp2, d_col2, d_cp, d_row, d_perm, t_ws, tws, NULL));
    GNN_CHECK(gnn_expand_ptr(N, q, d_rp2, d_erow, NULL));
    GNN_CHECK(gnn_expand_ptr(N, q, d_cp, d_ecol, NULL));
    gnn_graph_t graph;
    memset(&graph, 0, sizeof graph);
    graph.n = N; graph.nnz = q;
    graph.csr_rowptr = d_rp2; graph.csr_col = d_col2; graph.csr_erow = d_erow;
    graph.csc_colptr = d_cp; graph.csc_row = d_row; graph.csc_perm = d_perm; graph.csc_ecol = d_ecol;

    /* ---- the definition, dense and in double (row i attends to its stored entries j, self-loop included) ---- */
    static double Mm[N][F], sv[N][H], dv[N][H], al[H][N][N], rY[N * F], gy[H][N][N], ds[N][H], dd[N][H], dM[N][F];
    static double rdW[M * F], rdX[N * M], rdas[F], rdad[F], rdb[F];
    for (int i = 0; i < N; ++i) pat[i][i] = 1;
    for (int i = 0; i < N; ++i)
        for (int o = 0; o < F; ++o) { double s = 0; for (int c = 0; c < M; ++c) s += (double)X[i * M + c] * W[c * F + o]; Mm[i][o] = s; }
    for (int i = 0; i < N; ++i)
        for (int p = 0; p < H; ++p) {
            double s = 0, d = 0;
            for (int c = 0; c < KH; ++c) { s += as[p * KH + c] * Mm[i][p * KH + c]; d += ad[p * KH + c] * Mm[i][p * KH + c]; }
            sv[i][p] = s; dv[i][p] = d;
        }
    for (int p = 0; p < H; ++p)
        for (int i = 0; i < N; ++i) {
            double mx = -1e300, sum = 0;
            for (int j = 0; j < N; ++j) if (pat[i][j]) { double y = sv[i][p] + dv[j][p], w = y > 0 ? y : beta * y; if (w > mx) mx = w; }
            for (int j = 0; j < N; ++j) if (pat[i][j]) { double y = sv[i][p] + dv[j][p], w = y > 0 ? y : beta * y; al[p][i][j] = exp(w - mx); sum += al[p][i][j]; }
            for (int j = 0; j < N; ++j) al[p][i][j] = pat[i][j] ? al[p][i][j] / sum : 0.0;
            for (int c = 0; c < KH; ++c) {
                double s = b[p * KH + c];
                for (int j = 0; j < N; ++j) s += al[p][i][j] * Mm[j][p * KH + c];
                rY[i * F + p * KH + c] = s;
            }
        }
    for (int i = 0; i < N; ++i) for (int p = 0; p < H; ++p) { ds[i][p] = 0; dd[i][p] = 0; }
    for (int p = 0; p < H; ++p)
        for (int i = 0; i < N; ++i) {
            double t = 0;
            for (int j = 0; j < N; ++j) if (pat[i][j]) {
                double ga = 0;
                for (int c = 0; c < KH; ++c) ga += (double)G[i * F + p * KH + c] * Mm[j][p * KH + c];
                gy[p][i][j] = ga; t += al[p][i][j] * ga;
            }
            for (int j = 0; j < N; ++j) if (pat[i][j]) {
                double y = sv[i][p] + dv[j][p];
                gy[p][i][j] = al[p][i][j] * (gy[p][i][j] - t) * (y > 0 ? 1.0 : beta);
                ds[i][p] += gy[p][i][j]; dd[j][p] += gy[p][i][j];
            }
        }
    for (int j = 0; j < N; ++j)
        for (int p = 0; p < H; ++p)
            for (int c = 0; c < KH; ++c) {
                double s = ds[j][p] * as[p * KH + c] + dd[j][p] * ad[p * KH + c];
                for (int i = 0; i < N; ++i) s += al[p][i][j] * G[i * F + p * KH + c];
                dM[j][p * KH + c] = s;
            }
    for (int o = 0; o < F; ++o) {
        double a = 0, d = 0, g = 0;
        for (int i = 0; i < N; ++i) { a += ds[i][o / KH] * Mm[i][o]; d += dd[i][o / KH] * Mm[i][o]; g += G[i * F + o]; }
        rdas[o] = a; rdad[o] = d; rdb[o] = g;
    }
    for (int c = 0; c < M; ++c)
        for (int o = 0; o < F; ++o) { double s = 0; for (int i = 0; i < N; ++i) s += (double)X[i * M + c] * dM[i][o]; rdW[c * F + o] = s; }
    for (int i = 0; i < N; ++i)
        for (int c = 0; c < M; ++c) { double s = 0; for (int o = 0; o < F; ++o) s += dM[i][o] * W[c * F + o]; rdX[i * M + c] = s; }

    /* ---- every caching variant through the library ---- */
    float *d_X = dev_copy(X, sizeof X), *d_W = dev_copy(W, sizeof W), *d_as = dev_copy(as, sizeof as), *d_ad = dev_copy(ad, sizeof ad);
    float *d_b = dev_copy(b, sizeof b), *d_G = dev_copy(G, sizeof G), *d_Y = dev_copy(NULL, sizeof G);
    float *d_dW = dev_copy(NULL, sizeof W), *d_das = dev_copy(NULL, sizeof as), *d_dad = dev_copy(NULL, sizeof ad);
    float *d_db = dev_copy(NULL, sizeof b), *d_dX = dev_copy(NULL, sizeof X);
    if (!d_X || !d_W || !d_as || !d_ad || !d_b || !d_G || !d_Y || !d_dW || !d_das || !d_dad || !d_db || !d_dX) { fprintf(stderr, "device allocation failed\n"); return 2; }
    const gnn_cache_t variants[4] = {GNN_CACHE_NONE, GNN_CACHE_GAT_FEAT, GNN_CACHE_GAT_FEAT_NODEATT, GNN_CACHE_GAT_FEAT_EDGE};
    for (int v = 0; v < 4; ++v) {
        gnn_plan_desc_t desc;
        memset(&desc, 0, sizeof desc);
        desc.layer = GNN_LAYER_GAT; desc.n = N; desc.nnz = q; desc.f_in = M; desc.f_out = KH; desc.heads = H;
        desc.need_input_grad = 1; desc.has_bias = 1; desc.leaky_slope = beta; desc.cache = variants[v];
        gnn_plan_t *plan = NULL;
        gnn_plan_info_t info;
        GNN_CHECK(gnn_plan_create(&desc, &plan));
        GNN_CHECK(gnn_plan_query(plan, &info));
        void *ws = dev_copy(NULL, info.workspace_bytes), *cache = info.cache_bytes ? dev_copy(NULL, info.cache_bytes) : NULL;
        if (!ws || (info.cache_bytes && !cache)) { fprintf(stderr, "device allocation failed\n"); return 2; }
        GNN_CHECK(gat_layer_fwd(plan, &graph, d_X, d_W, d_as, d_ad, d_b, d_Y, cache, info.cache_bytes, ws,
                                info.workspace_bytes, NULL));
        GNN_CHECK(gat_layer_bwd(plan, &graph, d_X, d_W, d_as, d_ad, NULL, d_G, d_dW, d_das, d_dad, d_db, d_dX, cache,
                                info.cache_bytes, ws, info.workspace_bytes, NULL));
        HIP_OK(hipDeviceSynchronize());
        static float Y[N * F], dW[M * F], das[F], dad[F], db[F], dX[N * M];
        HIP_OK(hipMemcpy(Y, d_Y, sizeof Y, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dW, d_dW, sizeof dW, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(das, d_das, sizeof das, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dad, d_dad, sizeof dad, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(db, d_db, sizeof db, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dX, d_dX, sizeof dX, hipMemcpyDeviceToHost));
        int bad = compare("gat Y", Y, rY, N * F) | compare("gat dW", dW, rdW, M * F) | compare("gat da_src", das, rdas, F) |
                  compare("gat da_dst", dad, rdad, F) | compare("gat db", db, rdb, F) | compare("gat dX", dX, rdX, N * M);
        gnn_plan_destroy(plan);
        (void)hipFree(ws);
        if (cache) (void)hipFree(cache);
        if (bad) return 1;
        printf("ok: GAT layer from C, n=%d nnz=%d %d -> %d x %d, cache variant %d (%zu bytes)\n", N, (int)q, M, H, KH,
               (int)info.cache, info.cache_bytes);
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
    return gat_from_c();
}
