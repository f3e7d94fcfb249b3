// Element-wise kernels and tall column reductions (bias gradient, ReLU mask,
// attention-vector gradient, softmax cross-entropy).  All reductions are
// two-stage with a fixed summation order, so results are reproducible; they sum
// over every node, so they accumulate in double (a float sum of millions of
// terms of either sign is not accurate enough when the total is near zero).
#include "common.h"

namespace gnn {
namespace {

__global__ void __launch_bounds__(256)
activation_grad_kernel(long count4, long count, const float *__restrict__ G, const float *__restrict__ Y,
                       float *__restrict__ out, int vec, int act) {
    // derivative of the activation from its output y: ReLU 1 / 0, ELU 1 / y + 1 (= exp(x) for x <= 0)
    auto dact = [act](float g, float y) { return y > 0.f ? g : (act == kActElu ? g * (y + 1.f) : 0.f); };
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (vec) {
        if (i >= count4) return;
        const float4 g = reinterpret_cast<const float4 *>(G)[i];
        const float4 y = reinterpret_cast<const float4 *>(Y)[i];
        reinterpret_cast<float4 *>(out)[i] = make_float4(dact(g.x, y.x), dact(g.y, y.y), dact(g.z, y.z), dact(g.w, y.w));
    } else {
        if (i >= count) return;
        out[i] = dact(G[i], Y[i]);
    }
}

// Stage 1 of out[c] = sum_i wgt(i, c) * G[i][c].  A thread owns VEC consecutive columns; the 256
// threads of a block form (256 / fp) row lanes x fp column groups (fp = power of two >=
// min(f / VEC, 256)); each block owns `rows_per_block` consecutive rows and writes one partial
// row of f sums.  Four rows are in flight per thread (rotating accumulators, added in a
// fixed order).  VEC = 4 needs f and head_dim to be multiples of 4 and 16-byte aligned rows.
// With a second weight array wgt2 the kernel forms two sums in one launch: output columns [0, f) use wgt,
// columns [f, 2f) use wgt2 on the same G (the second read of a row comes from the cache); fo = 2f then.
template <int VEC>
__global__ void __launch_bounds__(256)
colsum_partial_kernel(long n, int f, int fo, int fp, long rows_per_block, const float *__restrict__ G,
                      const float *__restrict__ wgt, const float *__restrict__ wgt2, int heads, int head_dim,
                      const float *__restrict__ mask_y, int mask_act, double *__restrict__ part) {
    __shared__ double red[256][VEC];
    const int c0 = threadIdx.x % fp, rl = threadIdx.x / fp, lanes = 256 / fp;
    const long r0 = (long)blockIdx.x * rows_per_block;
    const long r1 = min(n, r0 + rows_per_block);
    const int groups = (fo + VEC - 1) / VEC;
    for (int cb = 0; cb < groups; cb += fp) {
        const int c = (cb + c0) * VEC;
        double a[4][VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < VEC; ++v) a[j][v] = 0.0;
        if (c < fo) {
            const int cg = c < f ? c : c - f;                         // column of G
            const float *wsel = c < f ? wgt : wgt2;
            const int hd = wsel ? cg / head_dim : 0;
            auto row = [&](long i, double (&acc)[VEC]) {
                const double w = wsel ? (double)wsel[(size_t)i * heads + hd] : 1.0;
                // with mask_y: G times the derivative of the fused activation, taken from its output
                auto dact = [mask_act](float g, float y) { return y > 0.f ? g : (mask_act == kActElu ? g * (y + 1.f) : 0.f); };
                if constexpr (VEC == 4) {
                    float4 g = *reinterpret_cast<const float4 *>(G + (size_t)i * f + cg);
                    if (mask_y) {
                        const float4 y = *reinterpret_cast<const float4 *>(mask_y + (size_t)i * f + cg);
                        g = make_float4(dact(g.x, y.x), dact(g.y, y.y), dact(g.z, y.z), dact(g.w, y.w));
                    }
                    acc[0] += w * g.x; acc[1] += w * g.y; acc[2] += w * g.z; acc[3] += w * g.w;
                } else {
                    float g = G[(size_t)i * f + cg];
                    if (mask_y) g = dact(g, mask_y[(size_t)i * f + cg]);
                    acc[0] += w * (double)g;
                }
            };
            long i = r0 + rl;
            for (; i + 3L * lanes < r1; i += 4L * lanes) {
                row(i, a[0]); row(i + lanes, a[1]); row(i + 2L * lanes, a[2]); row(i + 3L * lanes, a[3]);
            }
            for (; i < r1; i += lanes) row(i, a[0]);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) red[threadIdx.x][v] = (a[0][v] + a[1][v]) + (a[2][v] + a[3][v]);
        __syncthreads();
        if (rl == 0 && c < fo) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                double s = 0.0;
                for (int k = 0; k < lanes; ++k) s += red[k * fp + c0][v];
                part[(size_t)blockIdx.x * fo + c + v] = s;
            }
        }
        __syncthreads();
    }
}

// out[c] = sum over blocks of part[block][c].  A block of 256 threads covers 16 columns with
// 16 lanes each (lane j takes partials j, j+16, ... into four rotating accumulators); the
// lanes are then added in lane order, so the association is fixed.
// Columns [split, f) go to out2 (the second of two sums formed in one launch).
__global__ void __launch_bounds__(256)
colsum_final_kernel(int f, int split, int blocks, const double *__restrict__ part, float *__restrict__ out,
                    float *__restrict__ out2) {
    __shared__ double red[16][17];
    const int o = threadIdx.x % 16, sl = threadIdx.x / 16;
    const int c = blockIdx.x * 16 + o;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    if (c < f) {
        int b = sl;
        for (; b + 48 < blocks; b += 64) {
            a0 += part[(size_t)b * f + c];
            a1 += part[(size_t)(b + 16) * f + c];
            a2 += part[(size_t)(b + 32) * f + c];
            a3 += part[(size_t)(b + 48) * f + c];
        }
        for (; b < blocks; b += 16) a0 += part[(size_t)b * f + c];
    }
    red[sl][o] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (sl == 0 && c < f) {
        double t = 0.0;
        for (int k = 0; k < 16; ++k) t += red[k][o];
        if (c < split) out[c] = (float)t;
        else out2[c - split] = (float)t;
    }
}

// One thread per node: stable softmax, loss term, dZ = softmax - onehot.  Rows are read with a
// stride of c words between neighbouring threads; kept for rows too long for the tiled kernel.
__global__ void __launch_bounds__(256)
softmax_xent_rows_kernel(int n, int c, const float *__restrict__ Z, const int32_t *__restrict__ labels,
                         float *__restrict__ dZ, float *__restrict__ block_loss) {
    __shared__ float red[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    float loss = 0.f;
    if (i < n) {
        const float *z = Z + (size_t)i * c;
        float mx = z[0];
        for (int t = 1; t < c; ++t) mx = fmaxf(mx, z[t]);
        float sum = 0.f;
        for (int t = 0; t < c; ++t) sum += expf(z[t] - mx);
        const int lab = labels[i];
        loss = logf(sum) + mx - z[lab];
        const float inv = 1.f / sum;
        for (int t = 0; t < c; ++t) dZ[(size_t)i * c + t] = expf(z[t] - mx) * inv - (t == lab ? 1.f : 0.f);
    }
    red[threadIdx.x] = loss;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int k = 0; k < 256; ++k) s += red[k];
        block_loss[blockIdx.x] = s;
    }
}

constexpr int kXentLdsFloats = 12288;          // 48 KB tile of logits

// The same per 256-node block, tiled through LDS: a pass copies R = 256 / G whole rows (contiguous in
// memory, so the copy is coalesced), G = 2^g lanes share a row (elements lane, lane + G, ...; maximum and
// sum by a fixed xor tree), the gradients replace the logits in LDS and go out coalesced again.
__global__ void __launch_bounds__(256)
softmax_xent_tiled_kernel(int n, int c, int G, const float *__restrict__ Z, const int32_t *__restrict__ labels,
                          float *__restrict__ dZ, float *__restrict__ block_loss) {
    __shared__ float tile[kXentLdsFloats];
    __shared__ float red[256];
    const int R = 256 / G;
    const int r = threadIdx.x / G, g = threadIdx.x % G;
    const int first = blockIdx.x * 256;
    float loss = 0.f;
    for (int p0 = 0; p0 < 256 && first + p0 < n; p0 += R) {
        const int rows = min(R, n - first - p0);
        const size_t base = (size_t)(first + p0) * c;
        const int count = rows * c;
        for (int i = threadIdx.x; i < count; i += 256) tile[i] = Z[base + i];
        __syncthreads();
        float mx = -INFINITY, sum = 0.f, zl = 0.f;
        int lab = -1;
        float *z = tile + r * c;
        if (r < rows) {
            for (int t = g; t < c; t += G) mx = fmaxf(mx, z[t]);
            for (int o = G >> 1; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            for (int t = g; t < c; t += G) sum += expf(z[t] - mx);
            for (int o = G >> 1; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            lab = labels[first + p0 + r];
            zl = z[lab];
        }
        __syncthreads();                                   // every read of the logits precedes the overwrite
        if (r < rows) {
            if (g == 0) loss += logf(sum) + mx - zl;
            const float inv = 1.f / sum;
            for (int t = g; t < c; t += G) z[t] = expf(z[t] - mx) * inv - (t == lab ? 1.f : 0.f);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < count; i += 256) dZ[base + i] = tile[i];
        __syncthreads();
    }
    red[threadIdx.x] = loss;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int k = 0; k < 256; ++k) s += red[k];
        block_loss[blockIdx.x] = s;
    }
}

// out[0] = sum of `count` partials: thread t adds partials t, t + 256, ... in double, thread 0 adds the
// 256 results in order (a fixed association, whatever the count)
__global__ void __launch_bounds__(256)
sum_partials_kernel(int count, const float *__restrict__ in, float *__restrict__ out) {
    __shared__ double red[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) s += (double)in[i];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int k = 0; k < 256; ++k) t += red[k];
        out[0] = (float)t;
    }
}

// dZ = Z - T and one partial of 1/2 sum dZ^2 per block (grid-stride, fixed block count)
__global__ void __launch_bounds__(256)
squared_error_kernel(long count, const float *__restrict__ Z, const float *__restrict__ T, float *__restrict__ dZ,
                     float *__restrict__ block_loss) {
    __shared__ float red[256];
    float acc = 0.f;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long)gridDim.x * 256) {
        const float e = Z[i] - T[i];
        dZ[i] = e;
        acc = fmaf(0.5f * e, e, acc);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int k = 0; k < 256; ++k) s += red[k];
        block_loss[blockIdx.x] = s;
    }
}

long colsum_rows_per_block(long n) {
    long r = ceil_div(n, 1024);
    return r < 64 ? 64 : r;
}

}  // namespace

gnn_status_t activation_grad_launch(int64_t count, const float *G, const float *Y, float *out, int act, hipStream_t st) {
    if (count <= 0) return GNN_OK;
    const int vec = count % 4 == 0 && aligned16(G) && aligned16(Y) && aligned16(out);
    const long threads = vec ? count / 4 : count;
    hipLaunchKernelGGL(activation_grad_kernel, dim3((unsigned)ceil_div(threads, 256)), dim3(256), 0, st,
                       (long)(count / 4), (long)count, G, Y, out, vec, act);
    return launch_status();
}

size_t colsum_workspace_bytes(int64_t n, int f) {
    const long blocks = ceil_div(n > 0 ? n : 1, colsum_rows_per_block(n));
    return align_up((size_t)blocks * f * sizeof(double));
}

// out = sum_i wgt G (all of it when wgt is NULL); with wgt2 also out2 = sum_i wgt2 G from the same launch
static gnn_status_t colsum_weighted(int64_t n, int f, const float *G, const float *wgt, const float *wgt2, int heads,
                                    int head_dim, float *out, float *out2, void *workspace, hipStream_t st,
                                    const float *mask_y = nullptr, int mask_act = 0) {
    if (f <= 0) return GNN_OK;
    const long rpb = colsum_rows_per_block(n);
    const int blocks = (int)ceil_div(n > 0 ? n : 1, rpb);
    const bool vec = f % 4 == 0 && head_dim % 4 == 0 && aligned16(G) && (!mask_y || aligned16(mask_y));
    const int fo = wgt2 ? 2 * f : f;
    const int groups = vec ? fo / 4 : fo;
    int fp = 1;
    while (fp < groups && fp < 256) fp <<= 1;
    double *part = static_cast<double *>(workspace);
    if (vec)
        hipLaunchKernelGGL(colsum_partial_kernel<4>, dim3(blocks), dim3(256), 0, st, (long)n, f, fo, fp, rpb, G, wgt, wgt2,
                           heads, head_dim, mask_y, mask_act, part);
    else
        hipLaunchKernelGGL(colsum_partial_kernel<1>, dim3(blocks), dim3(256), 0, st, (long)n, f, fo, fp, rpb, G, wgt, wgt2,
                           heads, head_dim, mask_y, mask_act, part);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)ceil_div(fo, 16)), dim3(256), 0, st, fo, f, blocks, part, out,
                       out2);
    return launch_status();
}

gnn_status_t colsum_launch(int64_t n, int f, const float *G, float *out, void *workspace, hipStream_t st,
                           const float *mask_y, int mask_act) {
    return colsum_weighted(n, f, G, nullptr, nullptr, 1, f, out, nullptr, workspace, st, mask_y, mask_act);
}

gnn_status_t gat_attention_grad_launch(int n, int h, int k, const float *w, const float *M, float *da,
                                       void *workspace, hipStream_t st) {
    return colsum_weighted(n, h * k, M, w, nullptr, h, k, da, nullptr, workspace, st);
}

gnn_status_t gat_attention_grad2_launch(int n, int h, int k, const float *ds, const float *dd, const float *M,
                                        float *da_src, float *da_dst, void *workspace, hipStream_t st) {
    return colsum_weighted(n, h * k, M, ds, dd, h, k, da_src, da_dst, workspace, st);
}

gnn_status_t softmax_xent_launch(int n, int c, const float *Z, const int32_t *labels, float *dZ, float *loss,
                                 void *workspace, hipStream_t st) {
    if (n <= 0) return GNN_OK;
    const int blocks = (int)ceil_div(n, 256);
    float *part = static_cast<float *>(workspace);
    int G = 1;                                             // lanes per row: about 16 elements each
    while (G < 64 && G * 16 < c) G <<= 1;
    if ((long)(256 / G) * c <= kXentLdsFloats)
        hipLaunchKernelGGL(softmax_xent_tiled_kernel, dim3(blocks), dim3(256), 0, st, n, c, G, Z, labels, dZ, part);
    else
        hipLaunchKernelGGL(softmax_xent_rows_kernel, dim3(blocks), dim3(256), 0, st, n, c, Z, labels, dZ, part);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, blocks, part, loss);
    return launch_status();
}

gnn_status_t squared_error_launch(int64_t count, const float *Z, const float *T, float *dZ, float *loss,
                                  void *workspace, hipStream_t st) {
    float *part = static_cast<float *>(workspace);
    int blocks = (int)ceil_div(count > 0 ? count : 1, 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(squared_error_kernel, dim3(blocks), dim3(256), 0, st, (long)count, Z, T, dZ, part);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, blocks, part, loss);
    return launch_status();
}

}  // namespace gnn
