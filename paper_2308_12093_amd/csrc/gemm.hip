// fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32) for the tall-skinny
// products of the GCN / GAT layers:  X Theta,  G Theta^T  (rows = nodes, a few hundred
// columns at most) and  X^T H  (a small output reduced over all nodes).
//
// One block = 256 threads = 4 wavefronts arranged WM x WN; each wavefront owns
// TM x TN tiles of 32 x 32 outputs (16 accumulator registers per tile and lane).
// Both operands are staged through LDS k-major ([BK][rows + pad]) so that the
// operand reads of the matrix instruction are consecutive words; the loaders
// transpose on the way in when the source is stored the other way round.  The
// next k-tile is fetched into registers while the current one is multiplied.
//
// The transposed-A form splits the long reduction into `splits` chunks
// (blockIdx.y), writes one partial product per chunk and adds the partials in
// chunk order in a second kernel, so the result does not depend on scheduling.
//
// Block ids are remapped so that the eight XCDs (ids are dealt round-robin to
// them) each work on a contiguous range of tiles: column tiles of one row
// block, which re-read the same rows of A, share an L2.
#include "common.h"

namespace gnn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;

template <bool TA, bool TB, int WM, int WN, int TM, int TN>
__global__ void __launch_bounds__(256)
gemm_kernel(int M, int N, long K, const float *__restrict__ A, const float *__restrict__ B, float *__restrict__ C,
            const float *__restrict__ bias, int relu, long k_chunk, int tiles_m, int tiles_n, int vec_a, int vec_b) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int PA = TA ? 4 : 1, PB = TB ? 1 : 4;
    constexpr int GA = BM * BK / 4 / 256, GB = BN * BK / 4 / 256;   // float4 granules per thread
    __shared__ float As[BK][BM + PA];
    __shared__ float Bs[BK][BN + PB];

    const long total = (long)tiles_m * tiles_n;
    const long per_xcd = (total + 7) / 8;
    const long logical = (long)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= total) return;
    const int m0 = (int)(logical / tiles_n) * BM;
    const int n0 = (int)(logical % tiles_n) * BN;
    const long kbeg = (long)blockIdx.y * k_chunk;
    const long kend = min(K, kbeg + k_chunk);
    float *Cout = C + (size_t)blockIdx.y * (size_t)M * N;

    const int t = threadIdx.x;
    const int wave = t / 64, lane = t % 64;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane % 32, half = lane / 32;

    float4 ra[GA], rb[GB];

    auto fetch = [&](long k0) {
#pragma unroll
        for (int p = 0; p < GA; ++p) {
            const int j = t + 256 * p;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (!TA) {                           // A[M][K], granule runs along k
                const int row = j / (BK / 4), kq = (j % (BK / 4)) * 4;
                const long gi = m0 + row, gk = k0 + kq;
                if (gi < M) {
                    const float *src = A + gi * K + gk;
                    if (vec_a && gk + 3 < kend) v = *reinterpret_cast<const float4 *>(src);
                    else {
                        if (gk < kend) v.x = src[0];
                        if (gk + 1 < kend) v.y = src[1];
                        if (gk + 2 < kend) v.z = src[2];
                        if (gk + 3 < kend) v.w = src[3];
                    }
                }
            } else {                                       // A[K][M], granule runs along the output row index
                const int kk = j / (BM / 4), iq = (j % (BM / 4)) * 4;
                const long gk = k0 + kk, gi = m0 + iq;
                if (gk < kend) {
                    const float *src = A + gk * M + gi;
                    if (vec_a && gi + 3 < M) v = *reinterpret_cast<const float4 *>(src);
                    else {
                        if (gi < M) v.x = src[0];
                        if (gi + 1 < M) v.y = src[1];
                        if (gi + 2 < M) v.z = src[2];
                        if (gi + 3 < M) v.w = src[3];
                    }
                }
            }
            ra[p] = v;
        }
#pragma unroll
        for (int p = 0; p < GB; ++p) {
            const int j = t + 256 * p;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (!TB) {                           // B[K][N], granule runs along the output column index
                const int kk = j / (BN / 4), jq = (j % (BN / 4)) * 4;
                const long gk = k0 + kk, gj = n0 + jq;
                if (gk < kend) {
                    const float *src = B + gk * N + gj;
                    if (vec_b && gj + 3 < N) v = *reinterpret_cast<const float4 *>(src);
                    else {
                        if (gj < N) v.x = src[0];
                        if (gj + 1 < N) v.y = src[1];
                        if (gj + 2 < N) v.z = src[2];
                        if (gj + 3 < N) v.w = src[3];
                    }
                }
            } else {                                       // B[N][K], granule runs along k
                const int cj = j / (BK / 4), kq = (j % (BK / 4)) * 4;
                const long gj = n0 + cj, gk = k0 + kq;
                if (gj < N) {
                    const float *src = B + gj * K + gk;
                    if (vec_b && gk + 3 < kend) v = *reinterpret_cast<const float4 *>(src);
                    else {
                        if (gk < kend) v.x = src[0];
                        if (gk + 1 < kend) v.y = src[1];
                        if (gk + 2 < kend) v.z = src[2];
                        if (gk + 3 < kend) v.w = src[3];
                    }
                }
            }
            rb[p] = v;
        }
    };

    auto stage = [&]() {
#pragma unroll
        for (int p = 0; p < GA; ++p) {
            const int j = t + 256 * p;
            if constexpr (!TA) {
                const int row = j / (BK / 4), kq = (j % (BK / 4)) * 4;
                As[kq + 0][row] = ra[p].x; As[kq + 1][row] = ra[p].y;
                As[kq + 2][row] = ra[p].z; As[kq + 3][row] = ra[p].w;
            } else {
                const int kk = j / (BM / 4), iq = (j % (BM / 4)) * 4;
                *reinterpret_cast<float4 *>(&As[kk][iq]) = ra[p];
            }
        }
#pragma unroll
        for (int p = 0; p < GB; ++p) {
            const int j = t + 256 * p;
            if constexpr (!TB) {
                const int kk = j / (BN / 4), jq = (j % (BN / 4)) * 4;
                *reinterpret_cast<float4 *>(&Bs[kk][jq]) = rb[p];
            } else {
                const int cj = j / (BK / 4), kq = (j % (BK / 4)) * 4;
                Bs[kq + 0][cj] = rb[p].x; Bs[kq + 1][cj] = rb[p].y;
                Bs[kq + 2][cj] = rb[p].z; Bs[kq + 3][cj] = rb[p].w;
            }
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (kbeg < kend) {
        fetch(kbeg);
        stage();
        __syncthreads();
        for (long k0 = kbeg; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) fetch(k0 + BK);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                float a[TM], b[TN];
#pragma unroll
                for (int x = 0; x < TM; ++x) a[x] = As[kk + half][(wm * TM + x) * 32 + l32];
#pragma unroll
                for (int y = 0; y < TN; ++y) b[y] = Bs[kk + half][(wn * TN + y) * 32 + l32];
#pragma unroll
                for (int x = 0; x < TM; ++x)
#pragma unroll
                    for (int y = 0; y < TN; ++y)
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
            }
            __syncthreads();
            if (more) {
                stage();
                __syncthreads();
            }
        }
    }

    // accumulator register v of lane (half, l32) holds row 8*(v/4) + 4*half + v%4, column l32 of the tile
#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y) {
            const int gj = n0 + (wn * TN + y) * 32 + l32;
            if (gj >= N) continue;
            const float bj = bias ? bias[gj] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int gi = m0 + (wm * TM + x) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (gi < M) {
                    float o = acc[x][y][v] + bj;
                    if (relu) o = fmaxf(o, 0.f);
                    Cout[(size_t)gi * N + gj] = o;
                }
            }
        }
}

__global__ void __launch_bounds__(256)
splitk_reduce_kernel(long count, int splits, const float *__restrict__ part, float *__restrict__ C) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float a = 0.f;
    for (int s = 0; s < splits; ++s) a += part[(size_t)s * count + i];
    C[i] = a;
}

struct Tiling {
    int wm, wn, tm, tn;
    int bm() const { return wm * tm * 32; }
    int bn() const { return wn * tn * 32; }
};

Tiling pick_tiling(int64_t M, int64_t N) {
    if (M <= 64) return N <= 64 ? Tiling{2, 2, 1, 1} : Tiling{2, 2, 1, 2};
    if (N <= 32) return Tiling{4, 1, 1, 1};
    if (N <= 64) return Tiling{4, 1, 1, 2};
    return Tiling{2, 2, 2, 2};
}

// Number of chunks the reduction of a transposed-A product is cut into: enough blocks
// to fill the chip, as long as the partials stay a small fraction of the operand bytes.
int pick_splits(int ta, int64_t M, int64_t N, int64_t K) {
    if (!ta) return 1;
    const Tiling tl = pick_tiling(M, N);
    const int64_t tiles = ceil_div(M, tl.bm()) * ceil_div(N, tl.bn());
    int64_t s = 1024 / tiles;
    const int64_t by_k = K / (4 * BK);
    const int64_t by_traffic = K * (M + N) / (8 * M * N);
    if (s > by_k) s = by_k;
    if (s > by_traffic) s = by_traffic;
    if (s < 1) s = 1;
    return (int)s;
}

}  // namespace

size_t gemm_workspace_bytes(int ta, int tb, int64_t M, int64_t N, int64_t K) {
    (void)tb;
    const int s = pick_splits(ta, M, N, K);
    return s > 1 ? align_up((size_t)s * M * N * sizeof(float)) : kAlign;
}

#define GEMM_CASE(TA_, TB_, WM_, WN_, TM_, TN_)                                                                   \
    if (ta == TA_ && tb == TB_ && tl.wm == WM_ && tl.wn == WN_ && tl.tm == TM_ && tl.tn == TN_) {                 \
        hipLaunchKernelGGL((gemm_kernel<TA_, TB_, WM_, WN_, TM_, TN_>), grid, dim3(256), 0, st, (int)M, (int)N,   \
                           (long)K, A, B, out, splits > 1 ? nullptr : bias, splits > 1 ? 0 : relu, k_chunk,       \
                           tiles_m, tiles_n, vec_a, vec_b);                                                       \
        launched = true;                                                                                          \
    }
#define GEMM_TILINGS(TA_, TB_)                                                                          \
    GEMM_CASE(TA_, TB_, 2, 2, 1, 1) GEMM_CASE(TA_, TB_, 2, 2, 1, 2) GEMM_CASE(TA_, TB_, 4, 1, 1, 1)     \
    GEMM_CASE(TA_, TB_, 4, 1, 1, 2) GEMM_CASE(TA_, TB_, 2, 2, 2, 2)

gnn_status_t gemm_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, const float *B,
                         float *C, const float *bias, int relu, void *workspace, hipStream_t st) {
    if (M <= 0 || N <= 0) return GNN_OK;
    if (ta && tb) return GNN_ERR_UNSUPPORTED;
    if (M > INT32_MAX / 2 || N > INT32_MAX / 2) return GNN_ERR_UNSUPPORTED;
    const Tiling tl = pick_tiling(M, N);
    const int tiles_m = (int)ceil_div(M, tl.bm()), tiles_n = (int)ceil_div(N, tl.bn());
    const int splits = pick_splits(ta, M, N, K);
    long k_chunk = K;
    if (splits > 1) k_chunk = ceil_div(ceil_div(K, splits), BK) * BK;
    const int real_splits = splits > 1 ? (int)ceil_div(K, k_chunk) : 1;
    float *out = splits > 1 ? static_cast<float *>(workspace) : C;
    // a float4 may be read only if every granule start is 16-byte aligned
    const int vec_a = aligned16(A) && (ta ? M % 4 == 0 : K % 4 == 0);
    const int vec_b = aligned16(B) && (tb ? K % 4 == 0 : N % 4 == 0);
    const long total = (long)tiles_m * tiles_n;
    dim3 grid((unsigned)(8 * ceil_div(total, 8)), (unsigned)real_splits);
    bool launched = false;
    const bool TAb = ta != 0, TBb = tb != 0;
    if (!TAb && !TBb) { GEMM_TILINGS(false, false) }
    else if (!TAb && TBb) { GEMM_TILINGS(false, true) }
    else { GEMM_TILINGS(true, false) }
    if (!launched) return GNN_ERR_UNSUPPORTED;
    GNN_TRY(launch_status());
    if (splits > 1) {
        const long count = (long)M * N;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count,
                           real_splits, out, C);
        GNN_TRY(launch_status());
    }
    return GNN_OK;
}

}  // namespace gnn
