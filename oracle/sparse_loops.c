/*
 * fp64 CPU oracle, sparse part: plain loops over CSR arrays.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg can compare the HIP kernels with an independent, obviously correct
 * computation.  It shares no code, header, table or helper with the HIP
 * library.  Every routine is the defining loop nest of the operation, in
 * double precision, with no blocking, fusion or reordering; OpenMP only
 * splits an outer loop whose iterations write disjoint outputs.
 *
 * Index convention (App. D.1, read 0-based): rowptr[0] = 0, rowptr[n] = q,
 * row i owns slots rowptr[i] .. rowptr[i+1]-1 of col[] / val[].
 * Row i is the aggregating node, col[e] the neighbour it reads from.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- GCN preprocessing (Sec. "GCN Forward Pass": A^ = A + I, A' = D^-1/2 A^ D^-1/2) ---- */

/* Pattern of A^ = A + I: the diagonal entry of every row is present exactly
 * once (an existing one is kept, not doubled); columns stay ascending.
 * deg[i] = number of entries of row i of A^ (the row sum of the 0/1 matrix).
 * Returns the number of entries written. col_out must hold q + n entries. */
int64_t oracle_add_self_loops_degree(int32_t n, const int32_t *rowptr, const int32_t *col,
                                     int32_t *rowptr_out, int32_t *col_out, int32_t *deg)
{
    int64_t w = 0;
    for (int32_t i = 0; i < n; ++i) {
        rowptr_out[i] = (int32_t)w;
        int placed = 0;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int32_t j = col[e];
            if (!placed && j >= i) {
                if (j != i) col_out[w++] = i;
                placed = 1;
            }
            col_out[w++] = j;
        }
        if (!placed) col_out[w++] = i;
        deg[i] = (int32_t)(w - rowptr_out[i]);
    }
    rowptr_out[n] = (int32_t)w;
    return w;
}

/* A'_ij = A^_ij / sqrt(deg_i * deg_j), one value per stored entry. */
void oracle_gcn_normalize(int32_t n, const int32_t *rowptr, const int32_t *col,
                          const int32_t *deg, double *val)
{
#pragma omp parallel for schedule(dynamic, 1024)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
            val[e] = 1.0 / sqrt((double)deg[i] * (double)deg[col[e]]);
}

/* ---- CSR -> CSC (App. D.1: CSC = column pointers + row indices) ----
 * Counting sort of the row-major entry list by column.  It is stable, so the
 * rows inside a column come out ascending and the answer is unique.
 * perm[p] = CSR slot of the entry stored at CSC slot p. */
void oracle_csr_transpose(int32_t n, const int32_t *rowptr, const int32_t *col,
                          int32_t *colptr, int32_t *row_out, int32_t *perm)
{
    int32_t q = rowptr[n];
    memset(colptr, 0, sizeof(int32_t) * ((size_t)n + 1));
    for (int32_t e = 0; e < q; ++e) colptr[col[e] + 1]++;
    for (int32_t j = 0; j < n; ++j) colptr[j + 1] += colptr[j];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    memcpy(cursor, colptr, sizeof(int32_t) * (size_t)n);
    for (int32_t i = 0; i < n; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int32_t p = cursor[col[e]]++;
            row_out[p] = i;
            perm[p] = e;
        }
    free(cursor);
}

/* ---- SpMM, C = A B (App. E.1, the CSR row-gather loop; C starts at zero) ----
 * val == NULL means every stored entry is 1. */
void oracle_spmm(int32_t n, const int32_t *rowptr, const int32_t *col, const double *val,
                 const double *B, int32_t f, double *C)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n; ++i) {
        double *c = C + (size_t)i * f;
        for (int32_t t = 0; t < f; ++t) c[t] = 0.0;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const double *b = B + (size_t)col[e] * f;
            double v = val ? val[e] : 1.0;
            for (int32_t t = 0; t < f; ++t) c[t] += b[t] * v;
        }
    }
}

/* ---- C = A^T B by scattering over the CSR rows of A ----
 * C_j += A_ij B_i for every stored (i, j).  It never forms A^T, so it does not
 * depend on the transpose routine; it is the loop of the GCN listing in
 * App. G.1 (output[column] += features[i] * value).  The outer parallel loop
 * is over feature columns, so concurrent iterations write disjoint outputs. */
void oracle_spmm_transposed(int32_t n, const int32_t *rowptr, const int32_t *col, const double *val,
                            const double *B, int32_t f, double *C)
{
    memset(C, 0, sizeof(double) * (size_t)n * f);
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < f; ++t)
        for (int32_t i = 0; i < n; ++i)
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                C[(size_t)col[e] * f + t] += (val ? val[e] : 1.0) * B[(size_t)i * f + t];
}

/* ---- SDDMM, D = A .* (B C^T) on the pattern of A (App. E.2) ----
 * B is n x f, Ct is n x f (row j of Ct = column j of the paper's C), so
 * D_e = A_e * <B_i, Ct_j> for the entry e = (i, j).  val == NULL: A_e = 1. */
void oracle_sddmm(int32_t n, const int32_t *rowptr, const int32_t *col, const double *val,
                  const double *B, const double *Ct, int32_t f, double *D)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const double *b = B + (size_t)i * f, *c = Ct + (size_t)col[e] * f;
            double acc = 0.0;
            for (int32_t t = 0; t < f; ++t) acc += b[t] * c[t];
            D[e] = (val ? val[e] : 1.0) * acc;
        }
}

/* ==== GAT, per head (Sec. "GAT Forward Pass", "GAT Backward Pass") ====
 * Tensors with a head axis are [n][h][k] or [q][h]: head is the middle /
 * last axis.  Row i of the pattern is the node whose softmax runs over its
 * stored entries j (the set N(i) + {i}); s pairs with the row node, d with
 * the column node: y_ij = s_i + d_j. */

/* s_i = <a_src, m_i>, d_i = <a_dst, m_i> per head (App. B). */
void oracle_gat_node_attention(int32_t n, int32_t h, int32_t k, const double *M,
                               const double *a_src, const double *a_dst, double *s, double *d)
{
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = 0; p < h; ++p) {
            const double *m = M + ((size_t)i * h + p) * k;
            double ss = 0.0, dd = 0.0;
            for (int32_t c = 0; c < k; ++c) {
                ss += a_src[p * k + c] * m[c];
                dd += a_dst[p * k + c] * m[c];
            }
            s[(size_t)i * h + p] = ss;
            d[(size_t)i * h + p] = dd;
        }
}

/* Sign decision of LeakyReLU for the logit y = s + d.
 *   decide_fp32 != 0: both addends are rounded to float and added in float, the
 *     precision in which a kernel that was handed float s, d takes the decision;
 *   otherwise the decision is on the double y, except inside |y| <= tie_eps,
 *     where tie_mode > 0 counts the logit as positive and tie_mode < 0 as
 *     non-positive (tie_eps = 0: the plain rule y > 0). */
static int positive_logit(double s, double d, int decide_fp32, double tie_eps, int tie_mode)
{
    if (decide_fp32) {
        volatile float y = (float)s + (float)d;
        return y > 0.0f;
    }
    double y = s + d;
    if (tie_eps > 0.0 && fabs(y) <= tie_eps) return tie_mode > 0;
    return y > 0.0;
}

/* Edge logits, LeakyReLU (slope beta for y <= 0) and the softmax over each
 * row's stored entries.  The row maximum is subtracted before exp, which does
 * not change the quotient.  alpha and mask are [q][h]; mask = (y > 0). */
void oracle_gat_edge_softmax(int32_t n, int32_t h, const int32_t *rowptr, const int32_t *col,
                             const double *s, const double *d, double beta,
                             int decide_fp32, double tie_eps, int tie_mode,
                             double *alpha, uint8_t *mask)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = 0; p < h; ++p) {
            double mx = -INFINITY, sum = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double si = s[(size_t)i * h + p], dj = d[(size_t)col[e] * h + p];
                double y = si + dj;
                int pos = positive_logit(si, dj, decide_fp32, tie_eps, tie_mode);
                double w = pos ? y : beta * y;
                mask[(size_t)e * h + p] = (uint8_t)pos;
                alpha[(size_t)e * h + p] = w;
                if (w > mx) mx = w;
            }
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double x = exp(alpha[(size_t)e * h + p] - mx);
                alpha[(size_t)e * h + p] = x;
                sum += x;
            }
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) alpha[(size_t)e * h + p] /= sum;
        }
}

/* X'_{i,p,:} = sum_e alpha_{e,p} M_{col e,p,:}  (bias is added by the caller). */
void oracle_gat_aggregate(int32_t n, int32_t h, int32_t k, const int32_t *rowptr, const int32_t *col,
                          const double *alpha, const double *M, double *Y)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n; ++i) {
        double *y = Y + (size_t)i * h * k;
        for (int32_t t = 0; t < h * k; ++t) y[t] = 0.0;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const double *m = M + (size_t)col[e] * h * k;
            for (int32_t p = 0; p < h; ++p)
                for (int32_t c = 0; c < k; ++c) y[p * k + c] += alpha[(size_t)e * h + p] * m[p * k + c];
        }
    }
}

/* Backward over the edges:
 *   g_alpha_e = <G_i, M_j> per head          (the SDDMM, dL/dA = G M^T on the pattern)
 *   g_w_e     = alpha_e (g_alpha_e - sum_{u in row i} alpha_u g_alpha_u)   (softmax)
 *   g_y_e     = g_w_e * (mask_e ? 1 : beta)                                (LeakyReLU')
 *   ds_i      = sum over row i of g_y,  dd_j = sum over column j of g_y.
 * dd is accumulated serially per head, so no two threads touch one entry. */
void oracle_gat_edge_backward(int32_t n, int32_t h, int32_t k, const int32_t *rowptr, const int32_t *col,
                              const double *G, const double *M, const double *alpha, const uint8_t *mask,
                              double beta, double *gy, double *ds, double *dd)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = 0; p < h; ++p) {
            const double *g = G + ((size_t)i * h + p) * k;
            double t = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const double *m = M + ((size_t)col[e] * h + p) * k;
                double ga = 0.0;
                for (int32_t c = 0; c < k; ++c) ga += g[c] * m[c];
                gy[(size_t)e * h + p] = ga;
                t += alpha[(size_t)e * h + p] * ga;
            }
            double acc = 0.0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                size_t x = (size_t)e * h + p;
                double gw = alpha[x] * (gy[x] - t);
                gy[x] = gw * (mask[x] ? 1.0 : beta);
                acc += gy[x];
            }
            ds[(size_t)i * h + p] = acc;
        }
    memset(dd, 0, sizeof(double) * (size_t)n * h);
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < h; ++p)
        for (int32_t i = 0; i < n; ++i)
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                dd[(size_t)col[e] * h + p] += gy[(size_t)e * h + p];
}

/* dM_j = ds_j a_src + dd_j a_dst + sum_{e=(i,j)} alpha_e G_i   (A^T G by scatter). */
void oracle_gat_feature_grad(int32_t n, int32_t h, int32_t k, const int32_t *rowptr, const int32_t *col,
                             const double *alpha, const double *G, const double *ds, const double *dd,
                             const double *a_src, const double *a_dst, double *dM)
{
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < h; ++p) {
        for (int32_t j = 0; j < n; ++j)
            for (int32_t c = 0; c < k; ++c)
                dM[((size_t)j * h + p) * k + c] = ds[(size_t)j * h + p] * a_src[p * k + c]
                                                + dd[(size_t)j * h + p] * a_dst[p * k + c];
        for (int32_t i = 0; i < n; ++i)
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double a = alpha[(size_t)e * h + p];
                const double *g = G + ((size_t)i * h + p) * k;
                double *o = dM + ((size_t)col[e] * h + p) * k;
                for (int32_t c = 0; c < k; ++c) o[c] += a * g[c];
            }
    }
}

/* da[p][c] = sum_i w_{i,p} M_{i,p,c}   (dL/da_src with w = ds, dL/da_dst with w = dd). */
void oracle_gat_attention_grad(int32_t n, int32_t h, int32_t k, const double *w, const double *M, double *da)
{
    for (int32_t t = 0; t < h * k; ++t) da[t] = 0.0;
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = 0; p < h; ++p)
            for (int32_t c = 0; c < k; ++c)
                da[p * k + c] += w[(size_t)i * h + p] * M[((size_t)i * h + p) * k + c];
}

/* ---- softmax cross-entropy, summed over the nodes (the loss of the two-layer workload) ----
 * loss = sum_i ( log sum_c exp(Z_ic) - Z_{i,label_i} ),  dZ = softmax(Z) - onehot. */
double oracle_softmax_xent(int32_t n, int32_t c, const double *Z, const int32_t *label, double *dZ)
{
    double loss = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : loss)
    for (int32_t i = 0; i < n; ++i) {
        const double *z = Z + (size_t)i * c;
        double mx = z[0], sum = 0.0;
        for (int32_t t = 1; t < c; ++t) if (z[t] > mx) mx = z[t];
        for (int32_t t = 0; t < c; ++t) sum += exp(z[t] - mx);
        loss += log(sum) + mx - z[label[i]];
        for (int32_t t = 0; t < c; ++t)
            dZ[(size_t)i * c + t] = exp(z[t] - mx) / sum - (t == label[i] ? 1.0 : 0.0);
    }
    return loss;
}

int oracle_num_threads(void)
{
    int nt = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        nt = omp_get_num_threads();
    }
#endif
    return nt;
}
