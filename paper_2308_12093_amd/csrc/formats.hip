// SpMM in the other storage formats of App. D (coordinate, ELLPACK, hybrid) and the
// conversions from CSR, for the format comparison of App. E.1.  The layers do not use
// them: their SpMM is the entry-balanced CSR kernel.
//
// ELLPACK arrays are slot-major: slot j of row i lives at [j * n + i], so a wave that
// walks consecutive rows reads consecutive words.  Stored entries fill a row's slots
// from the front; the rest are padding (column -1, value 0).  The hybrid format keeps
// the first t entries of every row in ELLPACK arrays of width t and the remaining
// entries, row-major, in coordinate arrays (App. D.4).
#include "common.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace gnn {
namespace {

constexpr int kEllRows = 64;      // rows per block of the ELLPACK kernel
constexpr int kEllSlots = 16;     // slots staged per step
constexpr int kCooRun = 32;       // consecutive entries per lane group of the coordinate kernel
constexpr int kCooBatch = 8;      // of which this many gathers are in flight

// excess[i] = max(0, len_i - t), excess[n] = 0 (scanned afterwards); max_len = longest row
__global__ void __launch_bounds__(256)
hyb_count_kernel(int n, const int32_t *__restrict__ rowptr, int t, int32_t *__restrict__ excess,
                 int32_t *__restrict__ max_len) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    int len = 0;
    if (i < n) {
        len = rowptr[i + 1] - rowptr[i];
        excess[i] = len > t ? len - t : 0;
    } else if (i == n) {
        excess[n] = 0;
    }
    // one integer atomic per wave: the maximum does not depend on the order
    for (int o = 32; o > 0; o >>= 1) len = max(len, __shfl_xor(len, o));
    if ((threadIdx.x & 63) == 0 && len > 0) atomicMax(max_len, len);
}

// thread <-> (slot j, row i), rows fastest
__global__ void __launch_bounds__(256)
hyb_fill_ell_kernel(int n, int t, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                    const float *__restrict__ val, int32_t *__restrict__ ell_col, float *__restrict__ ell_val) {
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long)n * t) return;
    const int i = (int)(id % n), j = (int)(id / n);
    const int r0 = rowptr[i], len = rowptr[i + 1] - r0;
    const bool stored = j < len;
    ell_col[id] = stored ? col[r0 + j] : -1;
    ell_val[id] = stored ? (val ? val[r0 + j] : 1.f) : 0.f;
}

// one wave per row copies the entries beyond the first t
__global__ void __launch_bounds__(256)
hyb_fill_coo_kernel(int n, int t, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                    const float *__restrict__ val, const int32_t *__restrict__ rest_ptr,
                    int32_t *__restrict__ coo_row, int32_t *__restrict__ coo_col, float *__restrict__ coo_val) {
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (i >= n) return;
    const int r0 = rowptr[i] + t, r1 = rowptr[i + 1];
    const int o = rest_ptr[i];
    for (int e = r0 + lane; e < r1; e += 64) {
        coo_row[o + e - r0] = i;
        coo_col[o + e - r0] = col[e];
        coo_val[o + e - r0] = val ? val[e] : 1.f;
    }
}

__global__ void __launch_bounds__(256)
fill_zero_kernel(long count, float *__restrict__ p) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

__global__ void zero_word_kernel(int32_t *p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

// ELLPACK SpMM.  A block owns kEllRows consecutive rows and a tile of LANES * VEC features
// (blockIdx.y).  Per step it stages kEllSlots slots of its rows through LDS (coalesced
// along the rows); then every group of LANES threads walks the staged slots of its
// rows (row g, g + G, ...; G = 256 / LANES groups), one VEC-wide piece of B's row per lane.
// A step whose slots are all padding is skipped after the index read.
template <int LANES, int VEC>
__global__ void __launch_bounds__(256)
spmm_ell_kernel(int n, int t, const int32_t *__restrict__ ell_col, const float *__restrict__ ell_val,
                const float *__restrict__ B, int f, float *__restrict__ C) {
    constexpr int G = 256 / LANES;                  // lane groups per block
    constexpr int RPG = kEllRows / G;               // rows per group
    static_assert(RPG >= 1, "too few lanes per row");
    __shared__ int32_t s_col[kEllSlots][kEllRows];
    __shared__ float s_val[kEllSlots][kEllRows];

    const int row0 = blockIdx.x * kEllRows;
    const int g = threadIdx.x / LANES, lane = threadIdx.x % LANES;
    const int c0 = (blockIdx.y * LANES + lane) * VEC;
    const bool live = c0 < f;

    float acc[RPG][VEC];
#pragma unroll
    for (int r = 0; r < RPG; ++r)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[r][v] = 0.f;

    for (int j0 = 0; j0 < t; j0 += kEllSlots) {
        int any = 0;
#pragma unroll
        for (int k = 0; k < kEllSlots * kEllRows / 256; ++k) {
            const int id = k * 256 + threadIdx.x;
            const int sr = id % kEllRows, sj = id / kEllRows;
            int c = -1;
            float v = 0.f;
            if (row0 + sr < n && j0 + sj < t) {
                const size_t at = (size_t)(j0 + sj) * n + row0 + sr;
                c = ell_col[at];
                v = ell_val[at];
            }
            s_col[sj][sr] = c;
            s_val[sj][sr] = v;
            any |= c >= 0;
        }
        if (__syncthreads_or(any)) {
            if (live) {
#pragma unroll
                for (int r = 0; r < RPG; ++r) {
                    const int sr = g + r * G;
#pragma unroll
                    for (int sj = 0; sj < kEllSlots; sj += 4) {
                        if (s_col[sj][sr] < 0) break;           // stored entries come first in a row
                        float x[4][VEC], w[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {           // four gathers in flight
                            const int c = s_col[sj + u][sr];
                            w[u] = s_val[sj + u][sr];
#pragma unroll
                            for (int v = 0; v < VEC; ++v) x[u][v] = 0.f;
                            if (c >= 0) {
                                const float *b = B + (size_t)c * f + c0;
                                if constexpr (VEC == 4) {
                                    const float4 q = *reinterpret_cast<const float4 *>(b);
                                    x[u][0] = q.x; x[u][1] = q.y; x[u][2] = q.z; x[u][3] = q.w;
                                } else {
                                    x[u][0] = b[0];
                                }
                            }
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) acc[r][v] = fmaf(w[u], x[u][v], acc[r][v]);
                    }
                }
            }
        }
        __syncthreads();
    }
    if (!live) return;
#pragma unroll
    for (int r = 0; r < RPG; ++r) {
        const int i = row0 + g + r * G;
        if (i >= n) continue;
        float *out = C + (size_t)i * f + c0;
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4 *>(out) = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
        } else {
            out[0] = acc[r][0];
        }
    }
}

// Coordinate SpMM: C += A B, entry by entry (App. D.2).  A group of LANES threads takes
// kCooRun consecutive entries (in batches of kCooBatch gathers in flight) and a tile of
// LANES * VEC features; it adds up products while the row stays the same and sends the
// sum to C with floating-point atomics when the row changes, so sorted input costs one
// atomic per (row run, feature) and unsorted input still works.  The order of the atomic
// additions varies from run to run: the result is reproducible only up to fp32 rounding.
template <int LANES, int VEC>
__global__ void __launch_bounds__(256)
spmm_coo_kernel(long nnz, int run, const int32_t *__restrict__ row, const int32_t *__restrict__ col,
                const float *__restrict__ val, const float *__restrict__ B, int f, float *__restrict__ C) {
    constexpr int G = 256 / LANES;
    const int g = threadIdx.x / LANES, lane = threadIdx.x % LANES;
    const int c0 = (blockIdx.y * LANES + lane) * VEC;
    const long first = ((long)blockIdx.x * G + g) * run;
    if (c0 >= f || first >= nnz) return;
    const long end = min(first + run, nnz);

    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    auto flush = [&](int i) {
        float *out = C + (size_t)i * f + c0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            unsafeAtomicAdd(out + v, acc[v]);
            acc[v] = 0.f;
        }
    };
    int last = row[first];
    for (long e0 = first; e0 < end; e0 += kCooBatch) {
        const int cnt = (int)min((long)kCooBatch, end - e0);
        int r[kCooBatch], c[kCooBatch];
        float w[kCooBatch], x[kCooBatch][VEC];
#pragma unroll
        for (int k = 0; k < kCooBatch; ++k) {
            const long e = e0 + (k < cnt ? k : 0);
            r[k] = row[e];
            c[k] = col[e];
            w[k] = val ? val[e] : 1.f;
        }
#pragma unroll
        for (int k = 0; k < kCooBatch; ++k) {                // all gathers in flight before the first use
            const float *b = B + (size_t)c[k] * f + c0;
            if constexpr (VEC == 4) {
                const float4 q = *reinterpret_cast<const float4 *>(b);
                x[k][0] = q.x; x[k][1] = q.y; x[k][2] = q.z; x[k][3] = q.w;
            } else {
                x[k][0] = b[0];
            }
        }
#pragma unroll
        for (int k = 0; k < kCooBatch; ++k) {
            if (k < cnt) {
                if (r[k] != last) flush(last);
                last = r[k];
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = fmaf(w[k], x[k][v], acc[v]);
            }
        }
    }
    flush(last);
}

int pick_lanes(int f, int vec, int cap) {          // power of two >= f / vec, within [4, cap]
    int lanes = 4;
    while (lanes < cap && lanes * vec < f) lanes <<= 1;
    return lanes;
}

}  // namespace

gnn_status_t hyb_count_launch(int n, const int32_t *rowptr, int t, int32_t *rest_ptr, int32_t *max_len_dev,
                              void *scan_ws, hipStream_t st) {
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(64), 0, st, max_len_dev);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(hyb_count_kernel, dim3((unsigned)ceil_div((long)n + 1, 256)), dim3(256), 0, st, n, rowptr, t,
                       rest_ptr, max_len_dev);
    GNN_TRY(launch_status());
    return exclusive_scan_launch(rest_ptr, (long)n + 1, scan_ws, st);
}

gnn_status_t hyb_fill_launch(int n, int t, const int32_t *rowptr, const int32_t *col, const float *val,
                             const int32_t *rest_ptr, int32_t *ell_col, float *ell_val, int32_t *coo_row,
                             int32_t *coo_col, float *coo_val, hipStream_t st) {
    if (n <= 0) return GNN_OK;
    if (t > 0) {
        hipLaunchKernelGGL(hyb_fill_ell_kernel, dim3((unsigned)ceil_div((long)n * t, 256)), dim3(256), 0, st, n, t,
                           rowptr, col, val, ell_col, ell_val);
        GNN_TRY(launch_status());
    }
    if (rest_ptr) {
        hipLaunchKernelGGL(hyb_fill_coo_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, n, t, rowptr, col,
                           val, rest_ptr, coo_row, coo_col, coo_val);
        GNN_TRY(launch_status());
    }
    return GNN_OK;
}

gnn_status_t fill_zero_launch(int64_t count, float *p, hipStream_t st) {
    if (count <= 0) return GNN_OK;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, (long)count, p);
    return launch_status();
}

#define ELL_CASE(L, V)                                                                                          \
    if (lanes == L && vec == V) {                                                                               \
        hipLaunchKernelGGL((spmm_ell_kernel<L, V>), grid, dim3(256), 0, st, n, t, ell_col, ell_val, B, f, C);   \
        return launch_status();                                                                                 \
    }

gnn_status_t spmm_ell_launch(int n, int t, const int32_t *ell_col, const float *ell_val, const float *B, int f,
                             float *C, hipStream_t st) {
    if (n <= 0 || f <= 0) return GNN_OK;
    const int vec = f % 4 == 0 && aligned16(B) && aligned16(C) ? 4 : 1;
    const int lanes = pick_lanes(f, vec, 64);
    dim3 grid((unsigned)ceil_div(n, kEllRows), (unsigned)ceil_div(f, lanes * vec));
    ELL_CASE(4, 4) ELL_CASE(8, 4) ELL_CASE(16, 4) ELL_CASE(32, 4) ELL_CASE(64, 4)
    ELL_CASE(4, 1) ELL_CASE(8, 1) ELL_CASE(16, 1) ELL_CASE(32, 1) ELL_CASE(64, 1)
    return GNN_ERR_UNSUPPORTED;
}

#define COO_CASE(L, V)                                                                                          \
    if (lanes == L && vec == V) {                                                                               \
        dim3 grid((unsigned)ceil_div(nnz, (long)(256 / L) * run), (unsigned)ceil_div(f, L * V));                 \
        hipLaunchKernelGGL((spmm_coo_kernel<L, V>), grid, dim3(256), 0, st, (long)nnz, run, row, col, val, B,   \
                           f, C);                                                                               \
        return launch_status();                                                                                 \
    }

gnn_status_t spmm_coo_launch(int64_t nnz, const int32_t *row, const int32_t *col, const float *val, const float *B,
                             int f, float *C, hipStream_t st) {
    if (nnz <= 0 || f <= 0) return GNN_OK;
    const int vec = f % 4 == 0 && aligned16(B) ? 4 : 1;
    const int lanes = pick_lanes(f, vec, 32);
    const int run = kCooRun;      // shorter runs for small matrices were measured: more atomics, never faster
    COO_CASE(4, 4) COO_CASE(8, 4) COO_CASE(16, 4) COO_CASE(32, 4)
    COO_CASE(4, 1) COO_CASE(8, 1) COO_CASE(16, 1) COO_CASE(32, 1)
    return GNN_ERR_UNSUPPORTED;
}

}  // namespace gnn
