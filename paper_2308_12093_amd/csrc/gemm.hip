// Dense products of the GCN / GAT layers on the gfx950 matrix cores:
//   X Theta,  G Theta^T   rows = nodes, a few hundred columns at most   (fp32 MFMA)
//   X^T H                 a small output reduced over all nodes          (fp64 MFMA)
//
// One block = 256 threads = 4 wavefronts arranged WM x WN; each wavefront owns
// TM x TN output tiles of one matrix instruction (32 x 32 for
// v_mfma_f32_32x32x2_f32, 16 x 16 for v_mfma_f64_16x16x4_f64).  Operands are staged
// through LDS in the layout they have in memory, 16 bytes at a time.
//
// The transposed-A form  X^T H  sums over every node (up to millions of terms of
// either sign).  A float accumulator loses ~1e-7 * sqrt(#terms) * |term| there, which
// is above the accuracy asked of gradients whose value happens to be near zero, so
// that product runs on the fp64 matrix instruction: operands are widened from float
// when they leave LDS (their products are then exact) and accumulated in double.
// The reduction is split into chunks; each chunk writes one double partial and a
// second kernel adds the partials in chunk order, so the result does not depend on
// scheduling.
//
// Block ids are remapped so that the eight XCDs (ids are dealt round-robin to
// them) each work on a contiguous range of (chunk, tile) pairs: the tiles that
// re-read the same rows of an operand share an L2 and run close in time.
#include "common.h"

namespace gnn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef double doublex4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));   // a native vector: loads and stores stay typed

constexpr int kGemmGeneral = 0, kGemmInterior = 1, kGemmEdge = 2;

constexpr int BK = 32;

// ---- fp64: P[chunk][M][N] (double) = A[K][M]^T * B[K][N] over one chunk of K ---------------
// Both operands have the reduction index as their row index, so k-tiles go to LDS as they are
// ([BK][columns + pad], 16-byte in).  One v_mfma_f64_16x16x4_f64 takes, per lane (lu, lk), the
// element (k = lk, i = lu) of a 4 x 16 slice of each operand.  A wavefront owns TM x TN such
// tiles, interleaved: tile x holds the output rows  base + TM * i + x  (columns likewise with
// TN), so the TM values a lane needs from one k-row are consecutive words and come with one
// LDS read (b32 / b64 / b128), and the TN partial sums a lane holds for one output row are
// consecutive doubles.  Row padding spreads the four k-rows of a read over the banks.
// LDS is double-buffered: the next k-tile is fetched into registers before the current one is
// multiplied and written to the other buffer after it (one barrier per k-tile); the operands
// of k-step s+1 are read and widened before the instructions of step s.
// MASK: B is used as B .* act'(Ymask), the derivative of a fused activation taken from the layer's output
// Ymask (same shape as B): ReLU 1 / 0, ELU 1 / y + 1.  The gradient through the activation then needs no
// pass of its own: the second operand stream costs nothing while the matrix cores are the bound.
template <int WM, int WN, int TM, int TN, bool MASK>
__global__ void __launch_bounds__(256)
gemm_tn_f64_kernel(int M, int N, long K, const float *__restrict__ A, const float *__restrict__ B,
                   const float *__restrict__ Ymask, int mask_act,
                   double *__restrict__ P, long k_chunk, int tiles_m, int tiles_n, int splits, int vec_a, int vec_b) {
    constexpr int BM = WM * TM * 16, BN = WN * TN * 16, KSTEP = 4;
    // words per LDS row: the lanes of one k-row read 16 * T consecutive words; T = 1: four rows fill the 64
    // banks at a row length of 16 mod 64; T = 2: two rows per pass, 32 mod 64; T = 4: one row per pass
    constexpr int LA = BM + (TM == 1 ? (80 - BM % 64) % 64 : TM == 2 ? (96 - BM % 64) % 64 : 4);
    constexpr int LB = BN + (TN == 1 ? (80 - BN % 64) % 64 : TN == 2 ? (96 - BN % 64) % 64 : 4);
    constexpr int NA = BM * BK / 4, NB = BN * BK / 4;   // 16-byte granules per tile
    constexpr int GA = (NA + 255) / 256, GB = (NB + 255) / 256;
    extern __shared__ __align__(16) float lds[];
    float (*As)[BK][LA] = reinterpret_cast<float (*)[BK][LA]>(lds);                    // [2][BK][LA]
    float (*Bs)[BK][LB] = reinterpret_cast<float (*)[BK][LB]>(lds + 2 * BK * LA);      // [2][BK][LB]

    const long tiles = (long)tiles_m * tiles_n;
    const long total = tiles * splits;
    const long per_xcd = (total + 7) / 8;
    const long logical = (long)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= total) return;
    const int split = (int)(logical / tiles);
    const int tile = (int)(logical % tiles);
    const int m0 = (tile / tiles_n) * BM;
    const int n0 = (tile % tiles_n) * BN;
    const long kbeg = (long)split * k_chunk;
    const long kend = min(K, kbeg + k_chunk);

    const int t = threadIdx.x;
    const int wave = t / 64, lane = t % 64;
    const int wm = wave / WN, wn = wave % WN;
    const int lu = lane % 16, lk = lane / 16;           // position inside the instruction's operand

    floatx4 ra[GA], rb[GB];
    // granule j of a k-tile: k-row j / (cols / 4), columns 4 * (j % (cols / 4)) ...
    auto fetch_one = [&](const float *__restrict__ src, int cols_total, int col0, int tile_cols, int v4, long k0,
                         int j) __attribute__((always_inline)) {
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        const int kk = j / (tile_cols / 4), cq = (j % (tile_cols / 4)) * 4;
        const long gk = k0 + kk;
        const int gc = col0 + cq;
        if (gk < kend) {
            const float *q = src + gk * cols_total + gc;
            if (v4 && gc + 3 < cols_total) v = *reinterpret_cast<const floatx4 *>(q);
            else {
                if (gc < cols_total) v.x = q[0];
                if (gc + 1 < cols_total) v.y = q[1];
                if (gc + 2 < cols_total) v.z = q[2];
                if (gc + 3 < cols_total) v.w = q[3];
            }
        }
        return v;
    };
    auto fetch = [&](long k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < GA; ++p)
            if (NA % 256 == 0 || t + 256 * p < NA) ra[p] = fetch_one(A, M, m0, BM, vec_a, k0, t + 256 * p);
#pragma unroll
        for (int p = 0; p < GB; ++p)
            if (NB % 256 == 0 || t + 256 * p < NB) {
                rb[p] = fetch_one(B, N, n0, BN, vec_b, k0, t + 256 * p);
                if constexpr (MASK) {
                    const floatx4 y = fetch_one(Ymask, N, n0, BN, vec_b, k0, t + 256 * p);
                    auto dact = [mask_act](float g, float yy) { return yy > 0.f ? g : (mask_act == kActElu ? g * (yy + 1.f) : 0.f); };
                    rb[p] = floatx4{dact(rb[p].x, y.x), dact(rb[p].y, y.y), dact(rb[p].z, y.z), dact(rb[p].w, y.w)};
                }
            }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < GA; ++p) {
            const int j = t + 256 * p;
            if (NA % 256 == 0 || j < NA) *reinterpret_cast<floatx4 *>(&As[buf][j / (BM / 4)][(j % (BM / 4)) * 4]) = ra[p];
        }
#pragma unroll
        for (int p = 0; p < GB; ++p) {
            const int j = t + 256 * p;
            if (NB % 256 == 0 || j < NB) *reinterpret_cast<floatx4 *>(&Bs[buf][j / (BN / 4)][(j % (BN / 4)) * 4]) = rb[p];
        }
    };

    doublex4 acc[TM][TN];
#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y) acc[x][y] = doublex4{0.0, 0.0, 0.0, 0.0};

    auto read = [&](int buf, int kk, float (&av)[TM], float (&bv)[TN]) __attribute__((always_inline)) {
        const float *pa = &As[buf][kk + lk][(wm * 16 + lu) * TM];
        const float *pb = &Bs[buf][kk + lk][(wn * 16 + lu) * TN];
        if constexpr (TM == 4) { const floatx4 q = *reinterpret_cast<const floatx4 *>(pa); av[0] = q.x; av[1] = q.y; av[2] = q.z; av[3] = q.w; }
        else if constexpr (TM == 2) { const float2 q = *reinterpret_cast<const float2 *>(pa); av[0] = q.x; av[1] = q.y; }
        else av[0] = *pa;
        if constexpr (TN == 4) { const floatx4 q = *reinterpret_cast<const floatx4 *>(pb); bv[0] = q.x; bv[1] = q.y; bv[2] = q.z; bv[3] = q.w; }
        else if constexpr (TN == 2) { const float2 q = *reinterpret_cast<const float2 *>(pb); bv[0] = q.x; bv[1] = q.y; }
        else bv[0] = *pb;
    };
    auto mma = [&](const float (&av)[TM], const float (&bv)[TN]) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < TM; ++x)
#pragma unroll
            for (int y = 0; y < TN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)av[x], (double)bv[y], acc[x][y], 0, 0, 0);
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
        float a0[TM], b0[TN], a1[TM], b1[TN];
        read(buf, 0, a0, b0);
#pragma unroll
        for (int s2 = 0; s2 < BK / KSTEP; s2 += 2) {
            read(buf, (s2 + 1) * KSTEP, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (s2 + 2 < BK / KSTEP) read(buf, (s2 + 2) * KSTEP, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (kbeg < kend) {
        fetch(kbeg);
        stage(0);
        __syncthreads();
        int buf = 0;
        for (long k0 = kbeg; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) fetch(k0 + BK);
            multiply(buf);
            if (more) stage(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    // Accumulator register v of lane (lk, lu) of tile (x, y): row 4 v + lk, column lu of the 16 x 16 tile,
    // i.e. output row m0 + (wm * 16 + 4 v + lk) * TM + x, output column n0 + (wn * 16 + lu) * TN + y
    double *out = P + (size_t)split * M * N;
    const int gj0 = n0 + (wn * 16 + lu) * TN;
#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gi = m0 + (wm * 16 + 4 * v + lk) * TM + x;
            if (gi >= M) continue;
#pragma unroll
            for (int y = 0; y < TN; ++y)
                if (gj0 + y < N) out[(size_t)gi * N + gj0 + y] = acc[x][y][v];
        }
}

// ---- fp32: C[M][N] = A[M][K] * Bt[N][K]^T (+ bias, ReLU) --------------------------------
// Both operands have the reduction index contiguous in memory, so tiles go to LDS as they
// are ([rows][BK + 4], float4 in, float4 out).  One v_mfma_f32_32x32x2 multiplies a 32 x 2
// by a 2 x 32 slice; which two reduction indices those are is free as long as both operands
// agree, so the lower lane half takes k = 0..15 of the tile and the upper half k = 16..31:
// each lane then reads its 16 operand values of a tile row with four ds_read_b128.
//
// The layer products are tall and skinny (K is 16..512: a handful of k-tiles per output
// tile), so prologue and epilogue would dominate a one-tile-per-block kernel.  Blocks are
// persistent instead: each owns a contiguous range of output tiles and runs one software
// pipeline over all (tile, k-tile) steps of the range.  LDS is double-buffered; the global
// loads of step i+2 are issued before the matrix instructions of step i and written to LDS
// after those of step i+1 (one barrier per step), so the loads of the next output tile are
// in flight while the current tile is finished and stored.
//
// Three instantiations.  The two fast ones need 16-byte aligned operand rows (K a multiple of 4)
// and have no branch around a load in the step loop: the bias of the current tile is re-loaded
// every step, and the fetch cursor stops at the last step instead of being switched off (the
// last k-tile is simply read again), so the compiler counts outstanding loads exactly and waits
// only for the older of the two register sets.  kGemmInterior: M, N, K are multiples of the
// tile, every load is a uniform base plus a fixed lane offset.  kGemmEdge: any M, N, K; loads
// past an edge are redirected to valid addresses (see fetch).  kGemmGeneral guards every access
// (unaligned rows) and takes whatever waits that needs.

template <int WM, int WN, int TM, int TN, int BKT, int MODE>
__global__ void __launch_bounds__(256)
gemm_f32_kernel(int M, int N, int K, const float *__restrict__ A, const float *__restrict__ Bt,
                const float *__restrict__ A2, const float *__restrict__ Bt2, float *__restrict__ C, int ldc, const float *__restrict__ bias, int relu, int tiles_m, int tiles_n,
                int tiles_per_block, int vec_a, int vec_b) {
    constexpr bool FAST = MODE != kGemmGeneral;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = BKT, LD = BK + 4;
    constexpr int RPP = 256 / (BK / 4);                   // tile rows covered by one pass of the 256 threads
    constexpr int NJ = BK / 8;                            // 16-byte operand reads per tile row and lane
    constexpr int GA = (BM + RPP - 1) / RPP, GB = (BN + RPP - 1) / RPP;
    extern __shared__ __align__(16) float lds[];
    float (*As)[BM][LD] = reinterpret_cast<float (*)[BM][LD]>(lds);                    // [2][BM][LD]
    float (*Bs)[BN][LD] = reinterpret_cast<float (*)[BN][LD]>(lds + 2 * BM * LD);      // [2][BN][LD]

    // XCD-aware ownership: block ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous range of tiles, and each of its blocks a contiguous sub-range
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int xcd_first = xcd * per_xcd;
    const int xcd_last = min(total, xcd_first + per_xcd);
    const int first_tile = xcd_first + slot * tiles_per_block;
    const int last_tile = min(xcd_last, first_tile + tiles_per_block);
    if (first_tile >= last_tile) return;

    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t / 64), lane = t % 64;   // wave id as a scalar
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane % 32, half = lane / 32;
    // with a second operand pair the reduction runs over both: C = A Bt^T + A2 Bt2^T, kt1 k-tiles each
    const int kt1 = K > 0 ? (K + BK - 1) / BK : 1;
    const int ktiles = A2 ? 2 * kt1 : kt1;
    const int steps = (last_tile - first_tile) * ktiles;
    const int lrow = t / (BK / 4), lkq = (t % (BK / 4)) * 4;      // this thread's granule: row (+RPP per p), k offset
    // per-lane parts of the fast addresses, in bytes: address = wave-uniform base + 32-bit lane offset
    const unsigned lane_ld = ((unsigned)lrow * (unsigned)K + lkq) * 4u;
    const unsigned lane_st = ((unsigned)(4 * half) * (unsigned)ldc + l32) * 4u;

    // the loads of one (tile, k-tile) step, at a cursor that walks the block's steps in order.
    // Two register sets alternate, so the loads of step i+2 are issued before step i is
    // multiplied and have two steps of matrix work to arrive.
    floatx4 ra0[GA], rb0[GB], ra1[GA], rb1[GB];
    int ftm = first_tile / tiles_n, ftn = first_tile % tiles_n, fkt = 0, fstep = 0;
    auto guarded = [&](const float *__restrict__ src, int rows_total, int row0, int k0, int v4, floatx4 *reg,
                       int granules, int tile_rows) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < granules; ++p) {
            if (lrow + RPP * p >= tile_rows) continue;
            const long gr = row0 + lrow + RPP * p;
            const int gk = k0 + lkq;
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (gr < rows_total) {
                const float *q = src + gr * K + gk;
                if (v4 && gk + 3 < K) v = *reinterpret_cast<const floatx4 *>(q);
                else {
                    if (gk < K) v.x = q[0];
                    if (gk + 1 < K) v.y = q[1];
                    if (gk + 2 < K) v.z = q[2];
                    if (gk + 3 < K) v.w = q[3];
                }
            }
            reg[p] = v;
        }
    };
    bool kin0 = true, kin1 = true;                         // per register set: the lane's granule lies inside K
    auto fetch = [&](floatx4 (&ra)[GA], floatx4 (&rb)[GB], bool &kin) __attribute__((always_inline)) {
        const bool second = fkt >= kt1;                     // (never with one operand pair)
        const int m0 = ftm * BM, n0 = ftn * BN, k0 = (second ? fkt - kt1 : fkt) * BK;
        const float *Ao = second ? A2 : A, *Bo = second ? Bt2 : Bt;
        const float *pa = Ao + (size_t)m0 * K + k0;        // uniform bases of the tile being fetched
        const float *pb = Bo + (size_t)n0 * K + k0;
        if constexpr (FAST) {
            kin = true;
            if constexpr (MODE == kGemmInterior) {
                // every tile is full: one uniform base per load plus the lane's fixed offset
#pragma unroll
                for (int p = 0; p < GA; ++p)
                    if (BM % RPP == 0 || lrow + RPP * p < BM)
                        ra[p] = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const char *>(pa + (size_t)p * RPP * K) + lane_ld);
#pragma unroll
                for (int p = 0; p < GB; ++p)
                    if (BN % RPP == 0 || lrow + RPP * p < BN)
                        rb[p] = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const char *>(pb + (size_t)p * RPP * K) + lane_ld);
            } else {
                // ragged M, N or K: rows past the matrix re-read the last row (their products land in
                // accumulator rows that are never stored); a granule past K re-reads column 0 and is zeroed
                // on its way to LDS.  The same loads for every tile, none behind a branch, none out of bounds.
                const int gk = k0 + lkq;
                kin = gk < K;
                const float *ka = Ao + (kin ? gk : 0), *kb = Bo + (kin ? gk : 0);
#pragma unroll
                for (int p = 0; p < GA; ++p)
                    if (BM % RPP == 0 || lrow + RPP * p < BM)
                        ra[p] = *reinterpret_cast<const floatx4 *>(ka + (size_t)min(m0 + lrow + RPP * p, M - 1) * K);
#pragma unroll
                for (int p = 0; p < GB; ++p)
                    if (BN % RPP == 0 || lrow + RPP * p < BN)
                        rb[p] = *reinterpret_cast<const floatx4 *>(kb + (size_t)min(n0 + lrow + RPP * p, N - 1) * K);
            }
        } else {
            const bool kfull = k0 + BK <= K;
            if (kfull && vec_a && m0 + BM <= M && (size_t)BM * K < (1u << 30)) {
#pragma unroll
                for (int p = 0; p < GA; ++p)
                    if (BM % RPP == 0 || lrow + RPP * p < BM)
                        ra[p] = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const char *>(pa + (size_t)p * RPP * K) + lane_ld);
            } else {
                guarded(Ao, M, m0, k0, vec_a, ra, GA, BM);
            }
            if (kfull && vec_b && n0 + BN <= N && (size_t)BN * K < (1u << 30)) {
#pragma unroll
                for (int p = 0; p < GB; ++p)
                    if (BN % RPP == 0 || lrow + RPP * p < BN)
                        rb[p] = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const char *>(pb + (size_t)p * RPP * K) + lane_ld);
            } else {
                guarded(Bo, N, n0, k0, vec_b, rb, GB, BN);
            }
        }
        if (fstep + 1 < steps) {                           // the cursor stops at the last step
            ++fstep;
            if (++fkt == ktiles) {
                fkt = 0;
                if (++ftn == tiles_n) { ftn = 0; ++ftm; }
            }
        }
    };
    auto stage = [&](int buf, const floatx4 (&ra)[GA], const floatx4 (&rb)[GB], bool kin) __attribute__((always_inline)) {
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < GA; ++p)
            if (BM % RPP == 0 || lrow + RPP * p < BM)
                *reinterpret_cast<floatx4 *>(&As[buf][lrow + RPP * p][lkq]) = kin ? ra[p] : zero;
#pragma unroll
        for (int p = 0; p < GB; ++p)
            if (BN % RPP == 0 || lrow + RPP * p < BN)
                *reinterpret_cast<floatx4 *>(&Bs[buf][lrow + RPP * p][lkq]) = kin ? rb[p] : zero;
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // one k-tile in four quarters of eight reduction indices (four per lane half): the operand
    // reads of quarter j+1 are issued before the matrix instructions of quarter j (the scheduling
    // barriers keep that order), so LDS latency hides behind them
    static_assert(NJ == 4, "the quarter pipeline below is written for a k-tile of 32");
    auto read = [&](int buf, int j, floatx4 (&a)[TM], floatx4 (&b)[TN]) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < TM; ++x)
            a[x] = *reinterpret_cast<const floatx4 *>(&As[buf][(wm * TM + x) * 32 + l32][half * (BK / 2) + 4 * j]);
#pragma unroll
        for (int y = 0; y < TN; ++y)
            b[y] = *reinterpret_cast<const floatx4 *>(&Bs[buf][(wn * TN + y) * 32 + l32][half * (BK / 2) + 4 * j]);
    };
    auto quarter = [&](const floatx4 (&a)[TM], const floatx4 (&b)[TN]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y) {
                    const float av = c == 0 ? a[x].x : c == 1 ? a[x].y : c == 2 ? a[x].z : a[x].w;
                    const float bv = c == 0 ? b[y].x : c == 1 ? b[y].y : c == 2 ? b[y].z : b[y].w;
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[x][y], 0, 0, 0);
                }
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
        if (K <= 0) return;
        floatx4 a0[TM], b0[TN], a1[TM], b1[TN];
        read(buf, 0, a0, b0);
        read(buf, 1, a1, b1);
        __builtin_amdgcn_sched_barrier(0);
        quarter(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        read(buf, 2, a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        quarter(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
        read(buf, 3, a1, b1);
        __builtin_amdgcn_sched_barrier(0);
        quarter(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        quarter(a1, b1);
    };

    // write a finished output tile and clear the accumulators.
    // Accumulator register v of lane (half, l32): row 8*(v/4) + 4*half + v%4, column l32 of its 32 x 32 tile.
    int ctm = ftm, ctn = ftn, ckt = 0;                     // compute cursor
    // FAST: the bias of the tile being multiplied is (re)loaded at every step, ahead of that step's
    // operand loads and without a branch, so it has arrived by the time the step's LDS writes have
    // waited for the older register set: storing a finished tile then waits for no load at all.
    // (Without a bias any readable address serves; the value is discarded.)
    float bcol[TN];
    const float *bias_src = bias ? bias : Bt;
    auto load_bias = [&]() __attribute__((always_inline)) {
        if constexpr (FAST) {
#pragma unroll
            for (int y = 0; y < TN; ++y) bcol[y] = bias_src[min(ctn * BN + (wn * TN + y) * 32 + l32, N - 1)];
        }
    };
    auto finish_tile = [&]() __attribute__((always_inline)) {
        const int cm0 = ctm * BM, cn0 = ctn * BN;
        const bool cfull = cm0 + BM <= M && cn0 + BN <= N && (size_t)BM * ldc < (1u << 30);
        if (cfull) {
            float *c0 = C + (size_t)(cm0 + wm * TM * 32) * ldc + cn0 + wn * TN * 32;   // uniform per wavefront
            auto at = [&](int x, int y, int v) __attribute__((always_inline)) {
                return reinterpret_cast<float *>(reinterpret_cast<char *>(c0 + (size_t)(x * 32 + 8 * (v / 4) + (v % 4)) * ldc + y * 32) + lane_st);
            };
            auto put = [&](int x, int y, int v, float o) __attribute__((always_inline)) {
                // an output far larger than the caches is streamed past them
                if (relu & kActStream) __builtin_nontemporal_store(o, at(x, y, v));
                else *at(x, y, v) = o;
                acc[x][y][v] = 0.f;
            };
            if (!bias && !(relu & ~kActStream)) {
#pragma unroll
                for (int y = 0; y < TN; ++y)
#pragma unroll
                    for (int x = 0; x < TM; ++x)
#pragma unroll
                        for (int v = 0; v < 16; ++v) put(x, y, v, acc[x][y][v]);
            } else {
#pragma unroll
                for (int y = 0; y < TN; ++y) {
                    const float bj = FAST ? (bias ? bcol[y] : 0.f) : (bias ? bias[cn0 + (wn * TN + y) * 32 + l32] : 0.f);
#pragma unroll
                    for (int x = 0; x < TM; ++x) {
                        // what C holds, a whole 32 x 32 tile's worth of loads in flight before the first store
                        // (loads and stores go through the same pointer, so the compiler would not reorder them)
                        float held[16];
#pragma unroll
                        for (int v = 0; v < 16; ++v) held[v] = (relu & kActAccumulate) ? *at(x, y, v) : 0.f;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            float o = acc[x][y][v] + bj + held[v];
                            if (relu & kActRelu) o = fmaxf(o, 0.f);
                            put(x, y, v, o);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y) {
                    const int gj = cn0 + (wn * TN + y) * 32 + l32;
                    const float bj = FAST ? (bias ? bcol[y] : 0.f) : ((bias && gj < N) ? bias[gj] : 0.f);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int gi = cm0 + (wm * TM + x) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                        if (gj < N && gi < M) {
                            float o = acc[x][y][v] + bj;
                            if (relu & kActAccumulate) o += C[(size_t)gi * ldc + gj];
                            if (relu & kActRelu) o = fmaxf(o, 0.f);
                            C[(size_t)gi * ldc + gj] = o;
                        } else if (gj < ldc && gi < M) {
                            C[(size_t)gi * ldc + gj] = 0.f;           // padding columns of a wider row stride
                        }
                        acc[x][y][v] = 0.f;
                    }
                }
        }
        if (++ctn == tiles_n) { ctn = 0; ++ctm; }
    };
    auto after_multiply = [&]() __attribute__((always_inline)) {
        if (++ckt == ktiles) { ckt = 0; finish_tile(); }
    };

    // The pipeline fills inside the loop (two idle passes, steps -2 and -1, that only load and
    // stage), so the loop is entered with no load in flight and every pass sees the same state.
#pragma unroll
    for (int p = 0; p < GA; ++p) ra0[p] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < GB; ++p) rb0[p] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int step = -2; step < steps; step += 2) {
        // even step: multiply buffer 0; step+1 is in set 0, fetch step+2 into set 1
        load_bias();
        fetch(ra1, rb1, kin1);
        if (step >= 0) multiply(0);
        stage(1, ra0, rb0, kin0);
        __syncthreads();
        if (step >= 0) after_multiply();
        if (step + 1 >= steps) break;
        // odd step: multiply buffer 1; step+2 is in set 1, fetch step+3 into set 0
        load_bias();
        fetch(ra0, rb0, kin0);
        if (step >= 0) multiply(1);
        stage(0, ra1, rb1, kin1);
        __syncthreads();
        if (step >= 0) after_multiply();
    }
}

// out[c][r] = in[r][c] for a small weight matrix (rows x cols), through a 32 x 33 LDS tile.
__global__ void __launch_bounds__(256)
transpose_kernel(int rows, int cols, const float *__restrict__ in, float *__restrict__ out) {
    __shared__ float tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = in[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) out[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

// C[i] = sum over chunks of part[chunk][i].  A block covers 16 consecutive outputs with
// 16 chunk lanes each (lane j takes chunks j, j+16, ... into four rotating accumulators);
// the lanes are then added in lane order, so the association is fixed.
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(long count, int splits, const double *__restrict__ part, float *__restrict__ C) {
    __shared__ double red[16][17];
    const int o = threadIdx.x % 16, sl = threadIdx.x / 16;
    const long i = (long)blockIdx.x * 16 + o;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    if (i < count) {
        int s = sl;
        for (; s + 48 < splits; s += 64) {
            a0 += part[(size_t)s * count + i];
            a1 += part[(size_t)(s + 16) * count + i];
            a2 += part[(size_t)(s + 32) * count + i];
            a3 += part[(size_t)(s + 48) * count + i];
        }
        for (; s < splits; s += 16) a0 += part[(size_t)s * count + i];
    }
    red[sl][o] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (sl == 0 && i < count) {
        double t = 0.0;
        for (int k = 0; k < 16; ++k) t += red[k][o];
        C[i] = (float)t;
    }
}

struct Tiling {
    int wm, wn, tm, tn;
};

int tile_m(bool f64, const Tiling &t) { return t.wm * t.tm * (f64 ? 16 : 32); }
int tile_n(bool f64, const Tiling &t) { return t.wn * t.tn * (f64 ? 16 : 32); }

Tiling pick_tiling(bool f64, int64_t M, int64_t N) {
    if (f64) {
        if (N <= 16) return Tiling{4, 1, 1, 1};            // 64 x 16
        if (N <= 32) return Tiling{4, 1, 1, 2};            // 64 x 32
        if (M >= 256 && N >= 256) return Tiling{2, 2, 4, 4};   // 128 x 128
        return Tiling{2, 2, 2, 2};                         // 64 x 64
    }
    if (M <= 64) return N <= 64 ? Tiling{2, 2, 1, 1} : Tiling{2, 2, 1, 2};
    if (N <= 32) return Tiling{4, 1, 1, 1};
    if (N <= 64) return Tiling{4, 1, 1, 2};
    return Tiling{2, 2, 2, 2};
}

// Number of chunks the reduction of a transposed-A product is cut into: enough blocks
// to fill the chip, as long as the double partials (written and read once each) stay
// within a quarter of the operand bytes.
int pick_splits(int ta, int64_t M, int64_t N, int64_t K) {
    if (!ta) return 1;
    const Tiling tl = pick_tiling(true, M, N);
    const int64_t tiles = ceil_div(M, tile_m(true, tl)) * ceil_div(N, tile_n(true, tl));
    int64_t s = ceil_div(2048, tiles);
    const int64_t by_k = K / (4 * BK);
    const int64_t by_traffic = K * (M + N) / (16 * M * N);
    if (s > by_k) s = by_k;
    if (s > by_traffic) s = by_traffic;
    if (s < 1) s = 1;
    // equal blocks spread evenly over the 256 CUs only if their number is a multiple of 256: round down to one
    // (640 blocks leave half the CUs with three and half with two)
    if (tiles * s > 256) s = (tiles * s / 256 * 256) / tiles;
    return (int)s;
}

}  // namespace

size_t gemm_workspace_bytes(int ta, int tb, int64_t M, int64_t N, int64_t K) {
    if (!ta) return tb ? kAlign : align_up((size_t)(N > 0 ? N : 1) * (K > 0 ? K : 1) * sizeof(float));   // B^T
    return align_up((size_t)pick_splits(ta, M, N, K) * M * N * sizeof(double));
}

#define GEMM_F32_CASE(WM_, WN_, TM_, TN_)                                                                   \
    if (tl.wm == WM_ && tl.wn == WN_ && tl.tm == TM_ && tl.tn == TN_) {                                     \
        constexpr int BM_ = WM_ * TM_ * 32, BN_ = WN_ * TN_ * 32;                                           \
        const size_t lds = (size_t)2 * (BM_ + BN_) * (32 + 4) * sizeof(float);                              \
        const bool aligned = vec_a && vec_b && K > 0;                                                       \
        const bool interior = aligned && M % BM_ == 0 && N % BN_ == 0 && K % 32 == 0 &&                     \
                              (size_t)BM_ * K < (1u << 30) && (size_t)BN_ * K < (1u << 30) &&               \
                              (size_t)BM_ * ldc < (1u << 30);                                               \
        if (interior)                                                                                       \
            hipLaunchKernelGGL((gemm_f32_kernel<WM_, WN_, TM_, TN_, 32, kGemmInterior>), grid, dim3(256),   \
                               lds, st, (int)M, (int)N, (int)K, A, Bt, A2, Bt2, C, (int)ldc, bias, relu,      \
                               tiles_m, tiles_n, tiles_per_block, vec_a, vec_b);                            \
        else if (aligned)                                                                                   \
            hipLaunchKernelGGL((gemm_f32_kernel<WM_, WN_, TM_, TN_, 32, kGemmEdge>), grid, dim3(256), lds,  \
                               st, (int)M, (int)N, (int)K, A, Bt, A2, Bt2, C, (int)ldc, bias, relu,          \
                               tiles_m, tiles_n, tiles_per_block, vec_a, vec_b);                            \
        else                                                                                                \
            hipLaunchKernelGGL((gemm_f32_kernel<WM_, WN_, TM_, TN_, 32, kGemmGeneral>), grid, dim3(256),    \
                               lds, st, (int)M, (int)N, (int)K, A, Bt, A2, Bt2, C, (int)ldc, bias, relu,      \
                               tiles_m, tiles_n, tiles_per_block, vec_a, vec_b);                            \
        launched = true;                                                                                    \
    }
#define GEMM_F64_CASE(WM_, WN_, TM_, TN_)                                                                        \
    if (tl.wm == WM_ && tl.wn == WN_ && tl.tm == TM_ && tl.tn == TN_) {                                          \
        constexpr int BM_ = WM_ * TM_ * 16, BN_ = WN_ * TN_ * 16;                                                \
        constexpr int LA_ = BM_ + (TM_ == 1 ? (80 - BM_ % 64) % 64 : TM_ == 2 ? (96 - BM_ % 64) % 64 : 4);       \
        constexpr int LB_ = BN_ + (TN_ == 1 ? (80 - BN_ % 64) % 64 : TN_ == 2 ? (96 - BN_ % 64) % 64 : 4);       \
        const size_t lds = (size_t)2 * BK * (LA_ + LB_) * sizeof(float);                                         \
        if (b_mask)                                                                                              \
            hipLaunchKernelGGL((gemm_tn_f64_kernel<WM_, WN_, TM_, TN_, true>), grid, dim3(256), lds, st, (int)M,  \
                               (int)N, (long)K, A, B, b_mask, b_mask_act, static_cast<double *>(workspace),      \
                               k_chunk, tiles_m, tiles_n, splits, vec_a, vec_b);                                 \
        else                                                                                                     \
            hipLaunchKernelGGL((gemm_tn_f64_kernel<WM_, WN_, TM_, TN_, false>), grid, dim3(256), lds, st, (int)M, \
                               (int)N, (long)K, A, B, nullptr, 0, static_cast<double *>(workspace), k_chunk,     \
                               tiles_m, tiles_n, splits, vec_a, vec_b);                                          \
        launched = true;                                                                                         \
    }

gnn_status_t gemm_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, const float *B,
                         float *C, const float *bias, int relu, void *workspace, hipStream_t st,
                         const float *b_mask, int b_mask_act, int64_t ldc, const float *A2, const float *B2) {
    if (M <= 0 || N <= 0) return GNN_OK;
    if (ta && tb) return GNN_ERR_UNSUPPORTED;
    if ((A2 != nullptr) != (B2 != nullptr) || (A2 && ta)) return GNN_ERR_UNSUPPORTED;   // the plain products only
    // rows of C may be ldc >= N floats apart (the columns in between are written as zeros): the plain products only,
    // and few enough padding columns that the tiles covering N also cover them
    if (ldc == 0) ldc = N;
    if (ldc < N || ldc > (N + 31) / 32 * 32 || (ta && ldc != N) || ldc > INT32_MAX / 2) return GNN_ERR_UNSUPPORTED;
    if (b_mask && !ta) return GNN_ERR_UNSUPPORTED;         // only the transposed-A product masks its second operand
    if (M > INT32_MAX / 2 || N > INT32_MAX / 2 || (!ta && K > INT32_MAX / 2)) return GNN_ERR_UNSUPPORTED;
    const bool f64 = ta != 0;
    const Tiling tl = pick_tiling(f64, M, N);
    const int tiles_m = (int)ceil_div(M, tile_m(f64, tl)), tiles_n = (int)ceil_div(N, tile_n(f64, tl));
    bool launched = false;
    if (!f64) {
        // the kernel wants B with the reduction index contiguous: B[N][K]; transpose a [K][N] weight first
        const float *Bt = B, *Bt2 = B2;
        if (K <= 0) A2 = Bt2 = nullptr;                    // an empty reduction: nothing to add
        if (!tb && K > 0) {
            float *wt = static_cast<float *>(workspace);
            hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)ceil_div(N, 32), (unsigned)ceil_div(K, 32)), dim3(256),
                               0, st, (int)K, (int)N, B, wt);
            GNN_TRY(launch_status());
            Bt = wt;
            if (B2) {                                      // the second weight behind the first (2 x gemm_workspace_bytes)
                float *wt2 = reinterpret_cast<float *>(static_cast<char *>(workspace) + gemm_workspace_bytes(0, 0, M, N, K));
                hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)ceil_div(N, 32), (unsigned)ceil_div(K, 32)),
                                   dim3(256), 0, st, (int)K, (int)N, B2, wt2);
                GNN_TRY(launch_status());
                Bt2 = wt2;
            }
        }
        const int vec_a = aligned16(A) && (!A2 || aligned16(A2)) && K % 4 == 0;
        const int vec_b = aligned16(Bt) && (!Bt2 || aligned16(Bt2)) && K % 4 == 0;
        relu &= kActRelu | kActAccumulate;
        if ((size_t)M * N * sizeof(float) > kStreamBytes && !(relu & kActAccumulate)) relu |= kActStream;
        // persistent blocks: 64 per XCD (2 per CU), each owning a contiguous range of tiles
        const long total = (long)tiles_m * tiles_n;
        if (total > INT32_MAX / 4 || total * ceil_div(K > 0 ? K : 1, 32) > INT32_MAX / 4) return GNN_ERR_UNSUPPORTED;
        const long per_xcd = ceil_div(total, 8);
        const int blocks_per_xcd = (int)(per_xcd < 64 ? per_xcd : 64);
        const int tiles_per_block = (int)ceil_div(per_xcd, blocks_per_xcd);
        dim3 grid((unsigned)(8 * blocks_per_xcd));
        GEMM_F32_CASE(2, 2, 1, 1) GEMM_F32_CASE(2, 2, 1, 2) GEMM_F32_CASE(4, 1, 1, 1)
        GEMM_F32_CASE(4, 1, 1, 2) GEMM_F32_CASE(2, 2, 2, 2)
        if (!launched) return GNN_ERR_UNSUPPORTED;
        return launch_status();
    }
    int splits = pick_splits(ta, M, N, K);
    const long k_chunk = ceil_div(ceil_div(K > 0 ? K : 1, splits), BK) * BK;
    splits = (int)ceil_div(K > 0 ? K : 1, k_chunk);
    // a float4 may be read only if every granule start is 16-byte aligned
    const int vec_a = aligned16(A) && M % 4 == 0;
    const int vec_b = aligned16(B) && N % 4 == 0 && (!b_mask || aligned16(b_mask));
    const long total = (long)tiles_m * tiles_n * splits;
    dim3 grid((unsigned)(8 * ceil_div(total, 8)));
    GEMM_F64_CASE(4, 1, 1, 1) GEMM_F64_CASE(4, 1, 1, 2) GEMM_F64_CASE(2, 2, 2, 2) GEMM_F64_CASE(2, 2, 4, 4)
    if (!launched) return GNN_ERR_UNSUPPORTED;
    GNN_TRY(launch_status());
    const long count = (long)M * N;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)ceil_div(count, 16)), dim3(256), 0, st, count, splits,
                       static_cast<const double *>(workspace), C);
    return launch_status();
}

}  // namespace gnn
