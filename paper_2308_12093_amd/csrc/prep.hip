// Graph preprocessing: integer kernels (self-loops + degrees, CSR -> CSC, expansion of
// row pointers) and the symmetric normalisation  A' = D^-1/2 (A + I) D^-1/2
// (Sec. "GCN Forward Pass").  Every output is deterministic: integer atomics are
// only used for counts, and the CSC order comes from a stable radix sort.
#include "common.h"

namespace gnn {
namespace {

constexpr int SCAN_ITEMS = 4;                    // per thread
constexpr int SCAN_TILE = 256 * SCAN_ITEMS;

// Exclusive scan of one tile per block; block totals go to `sums` (if not NULL).
__global__ void __launch_bounds__(256)
scan_tile_kernel(long count, int32_t *__restrict__ data, int32_t *__restrict__ sums) {
    __shared__ int32_t wave_tot[4];
    const long base = (long)blockIdx.x * SCAN_TILE + (long)threadIdx.x * SCAN_ITEMS;
    int32_t v[SCAN_ITEMS];
    int32_t tsum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        v[i] = base + i < count ? data[base + i] : 0;
        tsum += v[i];
    }
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    int32_t incl = tsum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int32_t off = 0;
    for (int w = 0; w < wave; ++w) off += wave_tot[w];
    int32_t run = off + incl - tsum;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < count) data[base + i] = run;
        run += v[i];
    }
    if (sums && threadIdx.x == 255) sums[blockIdx.x] = off + incl;
}

__global__ void __launch_bounds__(256)
scan_add_kernel(long count, int32_t *__restrict__ data, const int32_t *__restrict__ sums) {
    const long i = (long)blockIdx.x * SCAN_TILE + threadIdx.x;
    const int32_t add = sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const long j = i + (long)k * 256;
        if (j < count) data[j] += add;
    }
}

gnn_status_t exclusive_scan_inplace(int32_t *data, long count, int32_t *ws, hipStream_t st) {
    if (count <= 0) return GNN_OK;
    const long blocks = ceil_div(count, SCAN_TILE);
    int32_t *sums = blocks > 1 ? ws : nullptr;
    hipLaunchKernelGGL(scan_tile_kernel, dim3((unsigned)blocks), dim3(256), 0, st, count, data, sums);
    GNN_TRY(launch_status());
    if (blocks > 1) {
        GNN_TRY(exclusive_scan_inplace(sums, blocks, ws + align_up(blocks * sizeof(int32_t)) / sizeof(int32_t), st));
        hipLaunchKernelGGL(scan_add_kernel, dim3((unsigned)blocks), dim3(256), 0, st, count, data, sums);
        GNN_TRY(launch_status());
    }
    return GNN_OK;
}

// ---- self-loops ---------------------------------------------------------------------
// new length of row i: one more unless the diagonal is already stored
__global__ void __launch_bounds__(256)
selfloop_count_kernel(int n, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                      int32_t *__restrict__ newlen, int32_t *__restrict__ deg) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i > n) return;
    if (i == n) { newlen[n] = 0; return; }
    int lo = rowptr[i], hi = rowptr[i + 1];
    const int len = hi - lo;
    while (lo < hi) {                               // first slot with col >= i
        const int mid = (lo + hi) >> 1;
        if (col[mid] < i) lo = mid + 1; else hi = mid;
    }
    const int has = lo < rowptr[i + 1] && col[lo] == i;
    newlen[i] = len + 1 - has;
    deg[i] = len + 1 - has;
}

// one wavefront per row: copy the row, inserting the diagonal at its sorted position
__global__ void __launch_bounds__(256)
selfloop_fill_kernel(int n, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                     const int32_t *__restrict__ rowptr_out, int32_t *__restrict__ col_out) {
    const int i = blockIdx.x * 4 + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    if (i >= n) return;
    const int s = rowptr[i], e = rowptr[i + 1], o = rowptr_out[i];
    const int grow = (rowptr_out[i + 1] - o) - (e - s);      // 1 if the diagonal has to be inserted
    int below = 0;                                           // entries with col < i seen by this lane
    for (int x = s + lane; x < e; x += 64) {
        const int c = col[x];
        below += c < i;
        col_out[o + (x - s) + (c > i ? grow : 0)] = c;
    }
    if (grow) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) below += __shfl_xor(below, d, 64);
        if (lane == 0) col_out[o + below] = i;
    }
}

__global__ void __launch_bounds__(256)
normalize_kernel(int n, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                 const int32_t *__restrict__ deg, float *__restrict__ val, int kind, float eps) {
    const int i = blockIdx.x * 4 + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    if (i >= n) return;
    const float di = (float)deg[i];
    for (int x = rowptr[i] + lane; x < rowptr[i + 1]; x += 64) {
        const int j = col[x];
        float v;
        if (kind == GNN_AGG_GCN_SYM) v = 1.0f / sqrtf(di * (float)deg[j]);
        else if (kind == GNN_AGG_MEAN) v = 1.0f / di;
        else v = j == i ? 1.0f + eps : 1.0f;
        val[x] = v;
    }
}

__global__ void __launch_bounds__(256)
expand_ptr_kernel(int n, const int32_t *__restrict__ ptr, int32_t *__restrict__ out) {
    const int i = blockIdx.x * 4 + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    if (i >= n) return;
    for (int x = ptr[i] + lane; x < ptr[i + 1]; x += 64) out[x] = i;
}

__global__ void __launch_bounds__(256)
gather_f32_kernel(long count, const float *__restrict__ in, const int32_t *__restrict__ perm, float *__restrict__ out) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) out[i] = in[perm[i]];
}

__global__ void __launch_bounds__(256)
gather_i32_kernel(long count, const int32_t *__restrict__ in, const int32_t *__restrict__ perm,
                  int32_t *__restrict__ out) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) out[i] = in[perm[i]];
}

// ---- CSR -> CSC ---------------------------------------------------------------------
__global__ void __launch_bounds__(256)
zero_i32_kernel(long count, int32_t *__restrict__ p) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0;
}

__global__ void __launch_bounds__(256)
column_count_kernel(long nnz, const int32_t *__restrict__ col, int32_t *__restrict__ counts) {
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e < nnz) atomicAdd(&counts[col[e]], 1);
}

constexpr int RADIX_ITEMS = 16;                    // keys per thread
constexpr int RADIX_TILE = 256 * RADIX_ITEMS;      // keys per block; wavefront w owns keys [w*1024, (w+1)*1024) of it

__global__ void __launch_bounds__(256)
radix_hist_kernel(long count, const int32_t *__restrict__ keys, int shift, int nblocks, int32_t *__restrict__ hist) {
    __shared__ int32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const long base = (long)blockIdx.x * RADIX_TILE;
#pragma unroll
    for (int r = 0; r < RADIX_ITEMS; ++r) {
        const long idx = base + r * 256 + threadIdx.x;
        if (idx < count) atomicAdd(&h[(keys[idx] >> shift) & 255], 1);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// Stable scatter of one tile.  `offs` holds, digit-major, the exclusive scan of the
// per-block digit counts.  Order inside a tile: wavefront, then round, then lane.
__global__ void __launch_bounds__(256)
radix_scatter_kernel(long count, const int32_t *__restrict__ keys, const int32_t *__restrict__ vals, int shift,
                     int nblocks, const int32_t *__restrict__ offs, int32_t *__restrict__ keys_out,
                     int32_t *__restrict__ vals_out) {
    __shared__ int32_t wbase[4][256];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    for (int w = 0; w < 4; ++w) wbase[w][threadIdx.x] = 0;
    __syncthreads();
    const long base = (long)blockIdx.x * RADIX_TILE + (long)wave * (64 * RADIX_ITEMS);
    int32_t k[RADIX_ITEMS];
#pragma unroll
    for (int r = 0; r < RADIX_ITEMS; ++r) {
        const long idx = base + r * 64 + lane;
        k[r] = idx < count ? keys[idx] : 0;
        if (idx < count) atomicAdd(&wbase[wave][(k[r] >> shift) & 255], 1);
    }
    __syncthreads();
    {                                               // digit = threadIdx.x: turn counts into start offsets per wavefront
        int32_t run = offs[(size_t)threadIdx.x * nblocks + blockIdx.x];
        for (int w = 0; w < 4; ++w) {
            const int32_t c = wbase[w][threadIdx.x];
            wbase[w][threadIdx.x] = run;
            run += c;
        }
    }
    __syncthreads();
    volatile int32_t *cnt = wbase[wave];
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < RADIX_ITEMS; ++r) {
        const long idx = base + r * 64 + lane;
        const bool valid = idx < count;
        const int digit = (k[r] >> shift) & 255;
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1;
            const unsigned long long bal = __ballot(valid && bit);
            same &= bit ? bal : ~bal;
        }
        const int rank = __popcll(same & below);
        const int total = __popcll(same);
        int32_t pos = 0;
        if (valid) pos = cnt[digit] + rank;
        __builtin_amdgcn_wave_barrier();
        if (valid && rank == total - 1) cnt[digit] = pos + 1;
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            keys_out[pos] = k[r];
            vals_out[pos] = vals ? vals[idx] : (int32_t)idx;
        }
    }
}

int radix_passes(int n) {
    int bits = 0;
    while ((1ll << bits) < (long long)n) ++bits;
    int p = (bits + 7) / 8;
    return p < 1 ? 1 : p;
}

size_t scan_ws_ints(long count) {
    size_t total = 0;
    long c = count;
    while (c > SCAN_TILE) {
        c = ceil_div(c, SCAN_TILE);
        total += align_up(c * sizeof(int32_t)) / sizeof(int32_t);
    }
    return total + kAlign / sizeof(int32_t);
}

}  // namespace

size_t scan_workspace_bytes(int64_t n) { return align_up(scan_ws_ints(n + 1) * sizeof(int32_t)); }

gnn_status_t exclusive_scan_launch(int32_t *data, long count, void *workspace, hipStream_t st) {
    return exclusive_scan_inplace(data, count, static_cast<int32_t *>(workspace), st);
}

gnn_status_t add_self_loops_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, int32_t *rowptr_out,
                                   int32_t *col_out, int32_t *deg_out, void *workspace, hipStream_t st) {
    (void)nnz;
    hipLaunchKernelGGL(selfloop_count_kernel, dim3((unsigned)ceil_div(n + 1, 256)), dim3(256), 0, st, n, rowptr, col,
                       rowptr_out, deg_out);
    GNN_TRY(launch_status());
    GNN_TRY(exclusive_scan_inplace(rowptr_out, (long)n + 1, static_cast<int32_t *>(workspace), st));
    if (n > 0) {
        hipLaunchKernelGGL(selfloop_fill_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, n, rowptr, col,
                           rowptr_out, col_out);
        GNN_TRY(launch_status());
    }
    return GNN_OK;
}

gnn_status_t normalize_launch(int n, const int32_t *rowptr, const int32_t *col, const int32_t *deg, float *val,
                              int kind, float eps, hipStream_t st) {
    if (n <= 0) return GNN_OK;
    hipLaunchKernelGGL(normalize_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, n, rowptr, col, deg, val,
                       kind, eps);
    return launch_status();
}

gnn_status_t expand_ptr_launch(int n, int nnz, const int32_t *ptr, int32_t *out, hipStream_t st) {
    (void)nnz;
    if (n <= 0) return GNN_OK;
    hipLaunchKernelGGL(expand_ptr_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, n, ptr, out);
    return launch_status();
}

gnn_status_t gather_f32_launch(int64_t count, const float *in, const int32_t *perm, float *out, hipStream_t st) {
    if (count <= 0) return GNN_OK;
    hipLaunchKernelGGL(gather_f32_kernel, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, (long)count, in,
                       perm, out);
    return launch_status();
}

// workspace layout: keys_b[nnz] | vals_b[nnz] | erow[nnz] | hist[256 * nblocks] | scan scratch
size_t transpose_workspace_bytes(int n, int nnz) {
    const long nblocks = ceil_div(nnz > 0 ? nnz : 1, RADIX_TILE);
    const long hist = 256 * nblocks;
    const long biggest_scan = hist > (long)n + 1 ? hist : (long)n + 1;
    return 3 * align_up((size_t)(nnz > 0 ? nnz : 1) * sizeof(int32_t)) + align_up(hist * sizeof(int32_t)) +
           align_up(scan_ws_ints(biggest_scan) * sizeof(int32_t));
}

gnn_status_t transpose_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, int32_t *colptr,
                              int32_t *row, int32_t *perm, void *workspace, hipStream_t st) {
    Carver ws(workspace);
    const long q = nnz;
    const long nblocks = ceil_div(q > 0 ? q : 1, RADIX_TILE);
    int32_t *keys_b = ws.take<int32_t>(q > 0 ? q : 1);
    int32_t *vals_b = ws.take<int32_t>(q > 0 ? q : 1);
    int32_t *erow = ws.take<int32_t>(q > 0 ? q : 1);
    int32_t *hist = ws.take<int32_t>(256 * nblocks);
    int32_t *scan_ws = reinterpret_cast<int32_t *>(ws.base + ws.off);

    // column pointers: histogram of the columns, then exclusive scan over n + 1 counters
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)ceil_div(n + 1, 256)), dim3(256), 0, st, (long)n + 1, colptr);
    GNN_TRY(launch_status());
    if (q > 0) {
        hipLaunchKernelGGL(column_count_kernel, dim3((unsigned)ceil_div(q, 256)), dim3(256), 0, st, q, col, colptr);
        GNN_TRY(launch_status());
    }
    GNN_TRY(exclusive_scan_inplace(colptr, (long)n + 1, scan_ws, st));
    if (q == 0) return GNN_OK;

    // stable LSD radix sort of the entry list by column; the payload is the CSR slot.
    // Buffers alternate so that the last pass lands in (row, perm).
    const int passes = radix_passes(n);
    const int32_t *kin = col, *vin = nullptr;
    for (int p = 0; p < passes; ++p) {
        const bool to_out = ((passes - 1 - p) % 2) == 0;
        int32_t *kout = to_out ? row : keys_b;
        int32_t *vout = to_out ? perm : vals_b;
        hipLaunchKernelGGL(radix_hist_kernel, dim3((unsigned)nblocks), dim3(256), 0, st, q, kin, 8 * p, (int)nblocks,
                           hist);
        GNN_TRY(launch_status());
        GNN_TRY(exclusive_scan_inplace(hist, 256 * nblocks, scan_ws, st));
        hipLaunchKernelGGL(radix_scatter_kernel, dim3((unsigned)nblocks), dim3(256), 0, st, q, kin, vin, 8 * p,
                           (int)nblocks, hist, kout, vout);
        GNN_TRY(launch_status());
        kin = kout;
        vin = vout;
    }
    // row index of every CSC slot: the row that owns CSR slot perm[p]
    GNN_TRY(expand_ptr_launch(n, nnz, rowptr, erow, st));
    hipLaunchKernelGGL(gather_i32_kernel, dim3((unsigned)ceil_div(q, 256)), dim3(256), 0, st, q, erow, perm, row);
    return launch_status();
}

}  // namespace gnn
