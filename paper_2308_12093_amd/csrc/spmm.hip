// CSR SpMM  C = A B  (App. E.1) for gfx950, with per-entry or per-(entry, head) weights.
//
// The operation is a gather of dense rows: bytes moved, not flops, bound it
// (operational intensity <= ~1 FLOP/byte, App. E.1).  Two things decide the
// achieved bandwidth on a graph with hubs: every lane must keep several
// independent row gathers in flight, and no lane group may own a whole hub row.
//
// Entry-balanced kernel (used when the expanded row index `erow` is given):
//   the entry list is cut into segments of `seg` consecutive entries; one group
//   of LPE lanes owns one segment, the lanes of the group spanning the feature
//   axis (VEC floats per lane and tile).  The group walks its entries U at a
//   time: it first issues the U index loads and the U dense-row gathers, none
//   of which depends on where rows begin or end, and only then folds them into
//   the accumulator, flushing it whenever erow changes.  Rows that lie inside
//   one segment are written straight to C.  A row cut by a segment boundary
//   leaves one partial per segment it touches in `part` (slot 2g: the row that
//   began before segment g; slot 2g+1: the row that continues after it), and a
//   second kernel adds the partials of each such row in segment order, so the
//   result does not depend on scheduling.
//
// Row kernel (no `erow`): one wavefront per row; same results, no balancing.
#include "common.h"

namespace gnn {
namespace {

__device__ __forceinline__ float epilogue(float x, const float *bias, int c, int relu) {
    if (bias) x += bias[c];
    if (relu) x = fmaxf(x, 0.f);
    return x;
}

template <int VEC>
__device__ __forceinline__ void store_row(float *dst, const float (&a)[VEC]) {
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(dst) = make_float4(a[0], a[1], a[2], a[3]);
    } else {
        dst[0] = a[0];
    }
}

template <int VEC, int LPE, int NT, int U, bool HEADS>
__global__ void __launch_bounds__(256)
spmm_seg_kernel(int nnz, int f, int seg, long nseg, const int32_t *__restrict__ erow,
                const int32_t *__restrict__ col, EdgeWeights w, const float *__restrict__ B,
                float *__restrict__ C, float *__restrict__ part, const float *__restrict__ bias, int relu) {
    constexpr int GPB = 256 / LPE;
    const int l = threadIdx.x % LPE;
    const long g = (long)blockIdx.x * GPB + threadIdx.x / LPE;
    if (g >= nseg) return;

    const int fbase = blockIdx.y * (LPE * VEC * NT);
    int foff[NT];
    bool fok[NT];
    int head[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        foff[t] = fbase + (t * LPE + l) * VEC;
        fok[t] = foff[t] < f;
        head[t] = HEADS ? (fok[t] ? foff[t] / w.head_dim : 0) : 0;
    }

    const int s = (int)(g * seg);
    const int e = min(nnz, s + seg);
    const int first = erow[s];
    const bool head_open = s > 0 && erow[s - 1] == first;

    float acc[NT][VEC];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[t][i] = 0.f;
    int cur = first;

    auto flush = [&](int row, bool to_head_slot, bool to_tail_slot) {
        float *dst;
        bool direct = false;
        if (to_head_slot) dst = part + (size_t)(2 * g) * f;
        else if (to_tail_slot) dst = part + (size_t)(2 * g + 1) * f;
        else { dst = C + (size_t)row * f; direct = true; }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (!fok[t]) continue;
            float o[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) o[i] = direct ? epilogue(acc[t][i], bias, foff[t] + i, relu) : acc[t][i];
            store_row<VEC>(dst + foff[t], o);
        }
    };

    for (int x = s; x < e; x += U) {
        int r[U], c[U];
        float v[U][NT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = min(x + u, e - 1);
            r[u] = erow[idx];
            c[u] = col[idx];
            const int slot = w.perm ? w.perm[idx] : idx;
            if (!w.val) {
#pragma unroll
                for (int t = 0; t < NT; ++t) v[u][t] = 1.f;
            } else if constexpr (HEADS) {
#pragma unroll
                for (int t = 0; t < NT; ++t) v[u][t] = w.val[(size_t)slot * w.heads + head[t]];
            } else {
                const float vv = w.val[slot];
#pragma unroll
                for (int t = 0; t < NT; ++t) v[u][t] = vv;
            }
        }
        float b[U][NT][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (fok[t]) {
                    const float *src = B + (size_t)c[u] * f + foff[t];
                    if constexpr (VEC == 4) {
                        const float4 q = *reinterpret_cast<const float4 *>(src);
                        b[u][t][0] = q.x; b[u][t][1] = q.y; b[u][t][2] = q.z; b[u][t][3] = q.w;
                    } else {
                        b[u][t][0] = *src;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) b[u][t][i] = 0.f;
                }
            }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (x + u < e) {
                if (r[u] != cur) {
                    flush(cur, cur == first && head_open, false);
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[t][i] = 0.f;
                    cur = r[u];
                }
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[t][i] = fmaf(v[u][t], b[u][t][i], acc[t][i]);
            }
        }
    }
    const bool tail_open = e < nnz && erow[e] == cur;
    const bool in_head = cur == first && head_open;
    flush(cur, in_head, !in_head && tail_open);
}

// Adds up, in segment order, the partials of every row that a segment boundary cuts.
template <int VEC>
__global__ void __launch_bounds__(256)
spmm_fixup_kernel(int nnz, int f, int seg, long nseg, const int32_t *__restrict__ erow,
                  const int32_t *__restrict__ rowptr, const float *__restrict__ part, float *__restrict__ C,
                  const float *__restrict__ bias, int relu) {
    const int fc = f / VEC;
    const long tid = (long)blockIdx.x * 256 + threadIdx.x;
    const long g = tid / fc;
    const int c = (int)(tid % fc) * VEC;
    if (g >= nseg) return;
    const long e = (g + 1) * seg;
    if (e >= nnz) return;                                  // nothing follows the last segment
    const int r = erow[e - 1];
    if (erow[e] != r) return;                              // the boundary falls between two rows
    const long s = g * seg;
    if (s > 0 && erow[s - 1] == r) return;                 // the row began earlier: its first segment owns it
    const long g_end = ((long)rowptr[r + 1] - 1) / seg;
    float a[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) a[i] = part[(size_t)(2 * g + 1) * f + c + i];
    for (long x = g + 1; x <= g_end; ++x)
#pragma unroll
        for (int i = 0; i < VEC; ++i) a[i] += part[(size_t)(2 * x) * f + c + i];
#pragma unroll
    for (int i = 0; i < VEC; ++i) C[(size_t)r * f + c + i] = epilogue(a[i], bias, c + i, relu);
}

// Rows without stored entries receive the epilogue of zero.
__global__ void __launch_bounds__(256)
spmm_empty_rows_kernel(int n, int f, const int32_t *__restrict__ rowptr, float *__restrict__ C,
                       const float *__restrict__ bias, int relu) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n || rowptr[i] != rowptr[i + 1]) return;
    for (int c = 0; c < f; ++c) C[(size_t)i * f + c] = epilogue(0.f, bias, c, relu);
}

// One wavefront per row, lanes stride over the features.
__global__ void __launch_bounds__(256)
spmm_row_kernel(int n, int f, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col, EdgeWeights w,
                const float *__restrict__ B, float *__restrict__ C, const float *__restrict__ bias, int relu) {
    const int row = blockIdx.x * 4 + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const int s = rowptr[row], e = rowptr[row + 1];
    for (int c = lane; c < f; c += kWave) {
        const int hd = w.heads > 1 ? c / w.head_dim : 0;
        float acc = 0.f;
        for (int x = s; x < e; ++x) {
            const int slot = w.perm ? w.perm[x] : x;
            const float v = w.val ? w.val[(size_t)slot * w.heads + hd] : 1.f;
            acc = fmaf(v, B[(size_t)col[x] * f + c], acc);
        }
        C[(size_t)row * f + c] = epilogue(acc, bias, c, relu);
    }
}

// profiling aid: events recorded right before / after the entry-balanced kernel
hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

int pow2_at_least(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

struct Shape {
    int vec, lpe, nt, tiles_y;
};

Shape pick_shape(int f, bool vec4) {
    Shape sh;
    sh.vec = vec4 ? 4 : 1;
    const int chunks = (f + sh.vec - 1) / sh.vec;          // VEC-wide chunks across the feature axis
    sh.lpe = pow2_at_least(chunks);
    if (sh.lpe > 64) sh.lpe = 64;
    if (!vec4 && sh.lpe < 8) sh.lpe = 8;
    int nt = (chunks + sh.lpe - 1) / sh.lpe;
    sh.nt = nt <= 1 ? 1 : (nt <= 2 ? 2 : 4);
    sh.tiles_y = (chunks + sh.lpe * sh.nt - 1) / (sh.lpe * sh.nt);
    return sh;
}

}  // namespace

// Segment length: as long as possible (fewer partials) while still giving the chip
// about eight wavefronts per SIMD (256 CUs x 4 SIMDs x 8 = 8192 wavefronts).
int spmm_segment_len(int64_t nnz, int f) {
    const Shape sh = pick_shape(f, f % 4 == 0);
    const int64_t groups_per_wave = kWave / sh.lpe;
    const int64_t want_groups = 8192 * groups_per_wave;
    int64_t seg = nnz / (want_groups > 0 ? want_groups : 1);
    int p = 16;
    while (p * 2 <= seg && p < 256) p <<= 1;
    return p;
}

size_t spmm_workspace_bytes(int64_t nnz, int f) {
    if (nnz <= 0) return kAlign;
    const int64_t nseg = ceil_div(nnz, spmm_segment_len(nnz, f));
    return align_up((size_t)(2 * nseg) * (size_t)f * sizeof(float));
}

#define SPMM_CASE(VEC_, LPE_, NT_, U_)                                                                       \
    if (sh.vec == VEC_ && sh.lpe == LPE_ && sh.nt == NT_) {                                                  \
        dim3 grid((unsigned)ceil_div(nseg, 256 / LPE_), (unsigned)sh.tiles_y);                               \
        if (heads)                                                                                           \
            hipLaunchKernelGGL((spmm_seg_kernel<VEC_, LPE_, NT_, U_, true>), grid, dim3(256), 0, st, nnz, f, \
                               seg, nseg, erow, col, w, B, C, part, bias, relu);                             \
        else                                                                                                 \
            hipLaunchKernelGGL((spmm_seg_kernel<VEC_, LPE_, NT_, U_, false>), grid, dim3(256), 0, st, nnz, f,\
                               seg, nseg, erow, col, w, B, C, part, bias, relu);                             \
        launched = true;                                                                                     \
    }

gnn_status_t spmm_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, const int32_t *erow,
                         EdgeWeights w, const float *B, int f, float *C, const float *bias, int relu,
                         void *workspace, hipStream_t st) {
    if (n <= 0 || f <= 0) return GNN_OK;
    if (w.heads < 1) w.heads = 1;
    if (w.heads == 1) w.head_dim = f;
    const bool heads = w.heads > 1 && w.val != nullptr;

    if (!erow || nnz == 0) {
        hipLaunchKernelGGL(spmm_row_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, n, f, rowptr, col, w,
                           B, C, bias, relu);
        return launch_status();
    }

    float *part = static_cast<float *>(workspace);
    const bool vec4 = f % 4 == 0 && aligned16(B) && aligned16(C) && aligned16(part) &&
                      (!heads || w.head_dim % 4 == 0);
    const Shape sh = pick_shape(f, vec4);
    const int seg = spmm_segment_len(nnz, f);
    const long nseg = ceil_div(nnz, seg);

    bool launched = false;
    if (g_prof_start) (void)hipEventRecord(g_prof_start, st);
    SPMM_CASE(4, 1, 1, 8) SPMM_CASE(4, 2, 1, 8) SPMM_CASE(4, 4, 1, 8) SPMM_CASE(4, 8, 1, 8)
    SPMM_CASE(4, 16, 1, 8) SPMM_CASE(4, 32, 1, 8) SPMM_CASE(4, 64, 1, 8) SPMM_CASE(4, 64, 2, 4)
    SPMM_CASE(4, 64, 4, 2)
    SPMM_CASE(1, 8, 1, 8) SPMM_CASE(1, 16, 1, 8) SPMM_CASE(1, 32, 1, 8) SPMM_CASE(1, 64, 1, 8)
    SPMM_CASE(1, 64, 2, 4) SPMM_CASE(1, 64, 4, 2)
    if (!launched) return GNN_ERR_UNSUPPORTED;
    if (g_prof_stop) (void)hipEventRecord(g_prof_stop, st);
    GNN_TRY(launch_status());

    const int vec = sh.vec;
    const long threads = nseg * (f / vec);
    if (vec == 4)
        hipLaunchKernelGGL(spmm_fixup_kernel<4>, dim3((unsigned)ceil_div(threads, 256)), dim3(256), 0, st, nnz, f, seg,
                           nseg, erow, rowptr, part, C, bias, relu);
    else
        hipLaunchKernelGGL(spmm_fixup_kernel<1>, dim3((unsigned)ceil_div(threads, 256)), dim3(256), 0, st, nnz, f, seg,
                           nseg, erow, rowptr, part, C, bias, relu);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(spmm_empty_rows_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, n, f, rowptr, C,
                       bias, relu);
    return launch_status();
}

void spmm_profile_events(hipEvent_t start, hipEvent_t stop) {
    g_prof_start = start;
    g_prof_stop = stop;
}

}  // namespace gnn
