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
//   axis (VEC floats per lane and tile); a 256-thread block owns GPB = 256 / LPE
//   consecutive segments (its "span").
//   1. The block copies erow, col and the weights of its span into LDS with
//      coalesced loads.
//   2. Each group walks its segment U entries at a time: wide LDS reads for the
//      indices, then U dense-row gathers issued back to back (they do not depend on
//      where rows begin or end), then the fold into the accumulator, which is
//      flushed whenever erow changes.  Rows that lie inside one segment are written
//      straight to C (bias / ReLU fused).
//   3. A row cut by a segment boundary leaves a partial in LDS (the row that began
//      before the segment: "head"; the row that continues after it: "tail").  After
//      a barrier the group that holds the tail of a row adds the heads of the
//      following segments of the block, in segment order, and writes the row.
//   4. Only rows that cross the block's span go to global memory: one head and one
//      tail partial per block, added in block order by spmm_fixup_kernel.
//   Every sum has a fixed association, so results are reproducible.
//
// Row kernel (no `erow`): one wavefront per row; same results, no balancing.
#include "common.h"

namespace gnn {
namespace {

__device__ __forceinline__ float epilogue(float x, const float *bias, int c, int act) {
    if (bias) x += bias[c];
    if (act == kActRelu) x = fmaxf(x, 0.f);
    else if (act == kActElu) x = x > 0.f ? x : expm1f(x);
    return x;
}

// four floats at a 4-byte aligned address: global dwordx4 accesses need no more than that
typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));

template <int N> struct IntVec;
template <> struct IntVec<8> { int4 a, b; __device__ int get(int i) const { const int4 &q = i < 4 ? a : b; i &= 3; return i == 0 ? q.x : i == 1 ? q.y : i == 2 ? q.z : q.w; } };
template <> struct IntVec<4> { int4 a; __device__ int get(int i) const { return i == 0 ? a.x : i == 1 ? a.y : i == 2 ? a.z : a.w; } };
template <> struct IntVec<2> { int2 a; __device__ int get(int i) const { return i == 0 ? a.x : a.y; } };

template <int N>
__device__ __forceinline__ IntVec<N> lds_read(const int32_t *p) {
    IntVec<N> v;
    if constexpr (N == 8) { v.a = *reinterpret_cast<const int4 *>(p); v.b = *reinterpret_cast<const int4 *>(p + 4); }
    else if constexpr (N == 4) v.a = *reinterpret_cast<const int4 *>(p);
    else v.a = *reinterpret_cast<const int2 *>(p);
    return v;
}

// per-segment bookkeeping kept in LDS for step 3
struct SegInfo {
    int32_t tail_row;      // row whose tail partial this segment holds, or -1
    int32_t has_head;      // the segment's first row began before it
    int32_t whole;         // ... and also continues after it (the segment is one slice of that row)
    int32_t active;        // the segment exists
};

// B has a row stride of ldb floats.  UA (VEC = 4 only) serves an f that is not a multiple of 4: B is then a
// copy padded to ldb = f rounded up (16-byte aligned rows, zeros in the padding), while the rows of C and
// `part` keep the stride f: whole groups of four go out as one 4-byte aligned 16-byte store, the lane that
// holds the ragged end of a row stores its one to three values one by one.
template <int VEC, int LPE, int NT, int U, bool HEADS, bool UA = false>
__global__ void __launch_bounds__(256)
spmm_seg_kernel(int nnz, int f, int ldb, int seg, long nseg, const int32_t *__restrict__ erow,
                const int32_t *__restrict__ col, EdgeWeights w, const float *__restrict__ B,
                float *__restrict__ C, float *__restrict__ part, const float *__restrict__ bias, int relu) {
    extern __shared__ __align__(16) int32_t smem[];
    constexpr int GPB = 256 / LPE;
    constexpr int FT = LPE * VEC * NT;                     // features handled by one block (blockIdx.y picks the tile)
    const int span = GPB * seg;
    int32_t *s_row = smem, *s_col = smem + span, *s_w = smem + 2 * span;
    float *s_head = reinterpret_cast<float *>(smem + 3 * span);          // [GPB][FT]
    float *s_tail = s_head + GPB * FT;                                  // [GPB][FT]
    SegInfo *s_info = reinterpret_cast<SegInfo *>(s_tail + GPB * FT);    // [GPB]

    const long blk_first = (long)blockIdx.x * span;
    for (int i = threadIdx.x; i < span; i += 256) {
        const long x = blk_first + i;
        if (x < nnz) {
            s_row[i] = erow[x];
            s_col[i] = col[x];
            const int slot = w.perm ? w.perm[x] : (int)x;
            if constexpr (HEADS) s_w[i] = slot;
            else s_w[i] = __float_as_int(w.val ? w.val[slot] : 1.f);
        }
    }
    __syncthreads();

    const int l = threadIdx.x % LPE;
    const int gl = threadIdx.x / LPE;                      // group inside the block
    const long g = (long)blockIdx.x * GPB + gl;
    const bool active = g < nseg;

    const int fbase = blockIdx.y * FT;
    int foff[NT], loff[NT];
    bool fok[NT];
    int head[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        loff[t] = (t * LPE + l) * VEC;                     // offset inside the block's feature tile
        foff[t] = fbase + loff[t];
        fok[t] = foff[t] < f;
        head[t] = HEADS ? (fok[t] ? foff[t] / w.head_dim : 0) : 0;
    }

    float acc[NT][VEC];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[t][i] = 0.f;

    auto store_lds = [&](float *dst) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if constexpr (VEC == 4)
                *reinterpret_cast<float4 *>(dst + loff[t]) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
            else dst[loff[t]] = acc[t][0];
        }
    };
    auto add_lds = [&](const float *src, bool overwrite) {   // acc (+)= src
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float q[VEC];
            if constexpr (VEC == 4) {
                const float4 v = *reinterpret_cast<const float4 *>(src + loff[t]);
                q[0] = v.x; q[1] = v.y; q[2] = v.z; q[3] = v.w;
            } else q[0] = src[loff[t]];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[t][i] = overwrite ? q[i] : acc[t][i] + q[i];
        }
    };
    auto store_global = [&](float *dst, bool with_epilogue) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (!fok[t]) continue;
            if constexpr (VEC == 4 && UA) {
                if (foff[t] + 4 <= f) {
                    float4u o;
                    o.x = with_epilogue ? epilogue(acc[t][0], bias, foff[t] + 0, relu) : acc[t][0];
                    o.y = with_epilogue ? epilogue(acc[t][1], bias, foff[t] + 1, relu) : acc[t][1];
                    o.z = with_epilogue ? epilogue(acc[t][2], bias, foff[t] + 2, relu) : acc[t][2];
                    o.w = with_epilogue ? epilogue(acc[t][3], bias, foff[t] + 3, relu) : acc[t][3];
                    *reinterpret_cast<float4u *>(dst + foff[t]) = o;
                } else {
#pragma unroll
                    for (int i = 0; i < 3; ++i)
                        if (foff[t] + i < f)
                            dst[foff[t] + i] = with_epilogue ? epilogue(acc[t][i], bias, foff[t] + i, relu) : acc[t][i];
                }
            } else if constexpr (VEC == 4) {
                float4 o;
                o.x = with_epilogue ? epilogue(acc[t][0], bias, foff[t] + 0, relu) : acc[t][0];
                o.y = with_epilogue ? epilogue(acc[t][1], bias, foff[t] + 1, relu) : acc[t][1];
                o.z = with_epilogue ? epilogue(acc[t][2], bias, foff[t] + 2, relu) : acc[t][2];
                o.w = with_epilogue ? epilogue(acc[t][3], bias, foff[t] + 3, relu) : acc[t][3];
                *reinterpret_cast<float4 *>(dst + foff[t]) = o;
            } else {
                dst[foff[t]] = with_epilogue ? epilogue(acc[t][0], bias, foff[t], relu) : acc[t][0];
            }
        }
    };
    auto clear = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[t][i] = 0.f;
    };

    SegInfo info{-1, 0, 0, active ? 1 : 0};
    if (active) {
        const int lb = gl * seg;                           // first LDS slot of this segment
        const long s = g * seg;
        const int cnt = (int)min((long)seg, (long)nnz - s);
        const int first = s_row[lb];
        const int before = gl > 0 ? s_row[lb - 1] : (s > 0 ? erow[s - 1] : -1);
        const bool head_open = before == first;
        int cur = first;

        auto batch = [&](const int (&r)[U], const int (&c)[U], const int (&wv)[U], int valid) {
            float v[U][NT];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    if constexpr (HEADS) v[u][t] = w.val[(size_t)wv[u] * w.heads + head[t]];
                    else v[u][t] = __int_as_float(wv[u]);
                }
            float b[U][NT][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    if (fok[t]) {
                        const float *src = B + (size_t)c[u] * ldb + foff[t];
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
                if (u < valid) {
                    if (r[u] != cur) {                     // the row `cur` ends here
                        if (cur == first && head_open) store_lds(s_head + gl * FT);
                        else store_global(C + (size_t)cur * f, true);
                        clear();
                        cur = r[u];
                    }
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[t][i] = fmaf(v[u][t], b[u][t][i], acc[t][i]);
                }
            }
        };

        int x = 0;
        for (; x + U <= cnt; x += U) {                     // full batches: wide LDS reads
            const IntVec<U> vr = lds_read<U>(s_row + lb + x), vc = lds_read<U>(s_col + lb + x),
                            vw = lds_read<U>(s_w + lb + x);
            int r[U], c[U], wv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) { r[u] = vr.get(u); c[u] = vc.get(u); wv[u] = vw.get(u); }
            batch(r, c, wv, U);
        }
        if (x < cnt) {                                     // ragged end of the entry list
            int r[U], c[U], wv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = lb + min(x + u, cnt - 1);
                r[u] = s_row[i]; c[u] = s_col[i]; wv[u] = s_w[i];
            }
            batch(r, c, wv, cnt - x);
        }
        // the last row of the segment
        const long e = s + cnt;
        const int after = e >= nnz ? -1 : (gl + 1 < GPB ? s_row[lb + seg] : erow[e]);
        const bool in_head = cur == first && head_open;
        info.has_head = head_open ? 1 : 0;
        if (in_head) {
            store_lds(s_head + gl * FT);
            info.whole = after == cur ? 1 : 0;
        } else if (after == cur) {
            store_lds(s_tail + gl * FT);
            info.tail_row = cur;
        } else {
            store_global(C + (size_t)cur * f, true);
        }
    }
    if (l == 0) s_info[gl] = info;
    __syncthreads();
    if (!active) return;

    // a row whose tail this segment holds: add the heads of the following segments of the block
    if (info.tail_row >= 0) {
        add_lds(s_tail + gl * FT, true);
        int x = gl + 1;
        bool open = true;                                  // the row still continues
        for (; x < GPB && s_info[x].active; ++x) {
            add_lds(s_head + x * FT, false);
            if (!s_info[x].whole) { open = false; break; }
        }
        if (open) store_global(part + (size_t)(2 * blockIdx.x + 1) * f, false);   // crosses the block's end
        else store_global(C + (size_t)info.tail_row * f, true);
    }
    // the row that began before the block: its slices inside this block, for the second kernel
    if (gl == 0 && info.has_head) {
        add_lds(s_head, true);
        for (int x = 0; s_info[x].whole && x + 1 < GPB && s_info[x + 1].active; ++x)
            add_lds(s_head + (x + 1) * FT, false);
        store_global(part + (size_t)(2 * blockIdx.x) * f, false);
    }
}

// Second kernel of the entry-balanced SpMM, one wavefront per block span b of the first:
//  (1) if a row starts in span b and continues past its end, add that row's
//      partials (slot 2b+1, then slot 2x of every later span x it reaches) and
//      write the row.  The 64 lanes form 64/LPF slots of LPF lanes; slot s takes the
//      partials b+1+s, b+1+s+slots, ... into four rotating accumulators, the slots
//      are then combined by a fixed shuffle tree: a hub row that spans hundreds of
//      blocks is summed in parallel, and always in the same order.
//  (2) lane i of wavefront w gives row 64 w + i the epilogue of zero if it is empty.
template <int VEC, bool RAGGED>                           // RAGGED: f is not a multiple of VEC
__global__ void __launch_bounds__(256)
spmm_fixup_kernel(int n, int nnz, int f, int span, long nspan, int lpf, const int32_t *__restrict__ erow,
                  const int32_t *__restrict__ rowptr, const float *__restrict__ part, float *__restrict__ C,
                  const float *__restrict__ bias, int relu) {
    const int lane = threadIdx.x % kWave;
    const long g = (long)blockIdx.x * 4 + threadIdx.x / kWave;

    const long row = g * kWave + lane;
    if (row < n && rowptr[row] == rowptr[row + 1])
        for (int c = 0; c < f; ++c) C[(size_t)row * f + c] = epilogue(0.f, bias, c, relu);

    if (g >= nspan) return;
    const long e = (g + 1) * span;
    if (e >= nnz) return;                                  // nothing follows the last span
    const int r = erow[e - 1];
    if (erow[e] != r) return;                              // the boundary falls between two rows
    const long s = g * span;
    if (s > 0 && erow[s - 1] == r) return;                 // the row began earlier: its first span owns it
    const long g_end = ((long)rowptr[r + 1] - 1) / span;

    const int fc = (f + VEC - 1) / VEC;                    // VEC-wide chunks of one row (the last may be ragged)
    const int slots = kWave / lpf, slot = lane / lpf, l = lane % lpf;
    for (int cb = 0; cb < fc; cb += lpf) {
        const int c = (cb + l) * VEC;
        const bool ok = cb + l < fc;
        float a[4][VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < VEC; ++i) a[j][i] = 0.f;
        if (ok) {
            long x = g + 1 + slot;
            for (; x + 3L * slots <= g_end; x += 4L * slots)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < VEC; ++i)
                        if (!RAGGED || c + i < f) a[j][i] += part[(size_t)(2 * (x + (long)j * slots)) * f + c + i];
            for (; x <= g_end; x += slots)                   // fewer than four left
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    if (!RAGGED || c + i < f) a[0][i] += part[(size_t)(2 * x) * f + c + i];
        }
        float t[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) t[i] = (a[0][i] + a[1][i]) + (a[2][i] + a[3][i]);
        for (int d = lpf; d < kWave; d <<= 1)
#pragma unroll
            for (int i = 0; i < VEC; ++i) t[i] += __shfl_xor(t[i], d, kWave);
        if (ok && slot == 0)
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!RAGGED || c + i < f)
                    C[(size_t)r * f + c + i] = epilogue(part[(size_t)(2 * g + 1) * f + c + i] + t[i], bias, c + i, relu);
    }
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

int pow2_at_least(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

struct Shape {
    int vec, lpe, nt, tiles_y;
};

// widths that are not a multiple of 4 (and wide enough to gain from it) run on a padded copy of B
bool padded_operand(int f) { return f % 4 != 0 && f > 4; }

// One thread per four consecutive columns of the padded copy (fp a multiple of 4, Bp 16-byte aligned).
__global__ void __launch_bounds__(256)
pad_rows_kernel(long n, int f, int fp, const float *__restrict__ B, float *__restrict__ Bp) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    const int q = fp / 4;
    if (i >= n * q) return;
    const long r = i / q;
    const int c = (int)(i - r * q) * 4;
    const float *src = B + r * f + c;
    float4 v;
    v.x = src[0];                                           // c < f always: fp - f < 4
    v.y = c + 1 < f ? src[1] : 0.f;
    v.z = c + 2 < f ? src[2] : 0.f;
    v.w = c + 3 < f ? src[3] : 0.f;
    *reinterpret_cast<float4 *>(Bp + r * fp + c) = v;
}

Shape pick_shape(int f, bool vec4) {
    Shape sh;
    sh.vec = vec4 ? 4 : 1;
    const int chunks = (f + sh.vec - 1) / sh.vec;          // VEC-wide chunks across the feature axis
    sh.lpe = pow2_at_least(chunks);
    if (sh.lpe > 64) sh.lpe = 64;
    if (!vec4 && sh.lpe < 8) sh.lpe = 8;
    int nt = (chunks + sh.lpe - 1) / sh.lpe;
    sh.nt = nt <= 1 ? 1 : 2;                               // wider rows take more feature tiles (grid.y)
    sh.tiles_y = (chunks + sh.lpe * sh.nt - 1) / (sh.lpe * sh.nt);
    return sh;
}

}  // namespace

// Segment length: as long as possible (fewer row cuts) while still giving the chip
// about eight wavefronts per SIMD (256 CUs x 4 SIMDs x 8 = 8192 wavefronts), and short
// enough that the index data of a block's segments fits a 24 KB LDS staging area.
int spmm_segment_len(int64_t nnz, int f) {
    const Shape sh = pick_shape(f, f % 4 == 0 || padded_operand(f));
    const int64_t groups_per_wave = kWave / sh.lpe;
    const int64_t want_groups = 8192 * groups_per_wave;
    const int64_t seg = nnz / (want_groups > 0 ? want_groups : 1);
    const int cap = 8 * sh.lpe < 256 ? 8 * sh.lpe : 256;   // (256 / lpe) groups x seg entries <= 2048
    int p = 16;
    while (p * 2 <= seg && p * 2 <= cap) p <<= 1;
    return p;
}

// Two partial rows per block of the first kernel.  The block count depends on whether the
// float4 path can be taken (pointer alignment is only known at launch): size for the larger.
static size_t partials_bytes(int64_t nnz, int f) {
    if (nnz <= 0) return kAlign;
    const int seg = spmm_segment_len(nnz, f);
    const int64_t span4 = (int64_t)(256 / pick_shape(f, f % 4 == 0 || padded_operand(f)).lpe) * seg;
    const int64_t span1 = (int64_t)(256 / pick_shape(f, false).lpe) * seg;
    const int64_t span = span4 < span1 ? span4 : span1;
    return align_up((size_t)(2 * ceil_div(nnz, span)) * (size_t)f * sizeof(float));
}

// ... followed, for a ragged width, by the padded copy of the dense operand
size_t spmm_workspace_bytes(int64_t n, int64_t nnz, int f) {
    size_t bytes = partials_bytes(nnz, f);
    if (padded_operand(f) && nnz > 0 && n > 0) bytes += align_up((size_t)n * ((f + 3) / 4 * 4) * sizeof(float));
    return bytes;
}

// Where spmm_launch puts the padded copy of B for this call, or NULL if the call makes none.
float *spmm_padded_operand(void *workspace, const int32_t *erow, int64_t b_rows, int64_t nnz, int f, int *ld) {
    if (!workspace || !erow || nnz <= 0 || b_rows <= 0 || !padded_operand(f)) return nullptr;
    if (ld) *ld = (f + 3) / 4 * 4;
    return reinterpret_cast<float *>(static_cast<char *>(workspace) + partials_bytes(nnz, f));
}

#define SPMM_CASE(VEC_, LPE_, NT_, U_)                                                                       \
    if (sh.vec == VEC_ && sh.lpe == LPE_ && sh.nt == NT_) {                                                  \
        constexpr int GPB_ = 256 / LPE_;                                                                     \
        dim3 grid((unsigned)ceil_div(nseg, GPB_), (unsigned)sh.tiles_y);                                     \
        const size_t lds = (size_t)3 * GPB_ * seg * sizeof(int32_t) +                                        \
                           (size_t)2 * GPB_ * (LPE_ * VEC_ * NT_) * sizeof(float) + GPB_ * sizeof(SegInfo);  \
        if (heads)                                                                                           \
            hipLaunchKernelGGL((spmm_seg_kernel<VEC_, LPE_, NT_, U_, true>), grid, dim3(256), lds, st, nnz,  \
                               f, f, seg, nseg, erow, col, w, B, C, part, bias, relu);                       \
        else if (VEC_ == 4 && ragged)                                                                        \
            hipLaunchKernelGGL((spmm_seg_kernel<VEC_, LPE_, NT_, U_, false, VEC_ == 4>), grid, dim3(256),    \
                               lds, st, nnz, f, fp, seg, nseg, erow, col, w, Bp, C, part, bias, relu);       \
        else                                                                                                 \
            hipLaunchKernelGGL((spmm_seg_kernel<VEC_, LPE_, NT_, U_, false>), grid, dim3(256), lds, st, nnz, \
                               f, f, seg, nseg, erow, col, w, B, C, part, bias, relu);                       \
        launched = true;                                                                                     \
    }

gnn_status_t spmm_launch(int n, int nnz, const int32_t *rowptr, const int32_t *col, const int32_t *erow,
                         EdgeWeights w, const float *B, long b_rows, int f, float *C, const float *bias, int relu,
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
    const bool aligned = f % 4 == 0 && aligned16(B) && aligned16(C) && aligned16(part);
    // a ragged width still takes four features per lane, on a padded copy of B (one weight per entry only:
    // a lane's four features must share a head)
    const bool ragged = padded_operand(f) && !heads && b_rows > 0;
    const bool vec4 = ragged || (aligned && (!heads || w.head_dim % 4 == 0));
    const Shape sh = pick_shape(f, vec4);
    const int fp = (f + 3) / 4 * 4;
    float *Bp = nullptr;
    if (ragged) {
        Bp = spmm_padded_operand(workspace, erow, b_rows, nnz, f, nullptr);
        if (B != Bp) {                                     // a caller that wrote the operand there itself: no copy
            hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)ceil_div(b_rows * (fp / 4), 256)), dim3(256), 0, st,
                               b_rows, f, fp, B, Bp);
            GNN_TRY(launch_status());
        }
    }
    const int seg = spmm_segment_len(nnz, f);
    const long nseg = ceil_div(nnz, seg);

    bool launched = false;
    SPMM_CASE(4, 1, 1, 8) SPMM_CASE(4, 2, 1, 8) SPMM_CASE(4, 4, 1, 8) SPMM_CASE(4, 8, 1, 8)
    SPMM_CASE(4, 16, 1, 8) SPMM_CASE(4, 32, 1, 8) SPMM_CASE(4, 64, 1, 8) SPMM_CASE(4, 64, 2, 4)
    SPMM_CASE(1, 8, 1, 8) SPMM_CASE(1, 16, 1, 8) SPMM_CASE(1, 32, 1, 8) SPMM_CASE(1, 64, 1, 8)
    SPMM_CASE(1, 64, 2, 4)
    if (!launched) return GNN_ERR_UNSUPPORTED;
    GNN_TRY(launch_status());

    // second kernel: one wavefront per block span of the first, and per 64 rows for the empty-row fill
    const int span = (256 / sh.lpe) * seg;
    const long nspan = ceil_div(nnz, span);
    int lpf = pow2_at_least((f + sh.vec - 1) / sh.vec);    // lanes per slot: one per VEC-wide chunk of a row
    if (lpf > kWave) lpf = kWave;
    const long waves = nspan > ceil_div(n, kWave) ? nspan : ceil_div(n, kWave);
    if (sh.vec == 4 && ragged)
        hipLaunchKernelGGL((spmm_fixup_kernel<4, true>), dim3((unsigned)ceil_div(waves, 4)), dim3(256), 0, st, n, nnz, f,
                           span, nspan, lpf, erow, rowptr, part, C, bias, relu);
    else if (sh.vec == 4)
        hipLaunchKernelGGL((spmm_fixup_kernel<4, false>), dim3((unsigned)ceil_div(waves, 4)), dim3(256), 0, st, n, nnz, f,
                           span, nspan, lpf, erow, rowptr, part, C, bias, relu);
    else
        hipLaunchKernelGGL((spmm_fixup_kernel<1, false>), dim3((unsigned)ceil_div(waves, 4)), dim3(256), 0, st, n, nnz, f,
                           span, nspan, lpf, erow, rowptr, part, C, bias, relu);
    return launch_status();
}

}  // namespace gnn
