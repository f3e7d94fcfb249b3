// Fused edge passes of the GAT layer (Eqs. gat-fwd-att, gat-fwd; Sec. "GAT Backward Pass") for gfx950.
//
// Every per-edge quantity of the layer is a function of a few per-node vectors (s, d, the softmax
// statistics of the row, t) and of the two feature rows the edge joins, so no per-edge array has to
// travel through memory between the steps.  Three passes over the stored entries do the whole edge
// phase, each with the entry-balanced work split of the SpMM (equal segments of the entry list, one
// group of lanes per segment, a lane owning four consecutive features of one head):
//
//   forward      (CSR)  Y_i = act(sum_e alpha_e M_j + b) with alpha the row softmax of
//                       LeakyReLU(s_i + d_j), as a running ("online") softmax: a lane keeps the
//                       running maximum m, the sum l of exp(w - m) and the weighted sum of its four
//                       features, and rescales both sums whenever the maximum grows.  Also writes the
//                       final (m, l) per (row, head), from which alpha_e = exp(w_e - m) / l later.
//   backward row (CSR)  g_alpha_e = <G_i, M_j> per head (the SDDMM), folded at once into the three
//                       row sums t = sum alpha g_alpha, P = sum_{y>0} alpha g_alpha, Q = sum_{y>0} alpha;
//                       ds_i = (1 - beta)(P - t Q) because the softmax gradient sums to zero over a row.
//                       Without cached alpha the sums are taken over exp(w - m) with a running maximum,
//                       like the forward pass, and divided by l at the end: no separate statistics pass.
//   backward col (CSC)  recomputes g_alpha_e from G_i (gathered anyway for A^T G) and M_j (the
//                       column's own row), g_y_e = alpha_e (g_alpha_e - t_i) f'(y_e), and accumulates
//                       dd_j = sum g_y and dM_j = sum alpha_e G_i; the rank-one terms ds_j a_src +
//                       dd_j a_dst are added when the row is written.
//
// alpha and the LeakyReLU sign come from the cache when the variant keeps them (read in entry order by the
// row pass, through perm by the column pass; having the row pass leave them as one signed value per entry
// and head, to halve the column pass's gathers, cost more in scattered writes than it saved).
// Otherwise they are rebuilt per entry from per-node values: s_i, d_j and the row statistics - the same
// arithmetic on the same bits in every pass, so all passes see the same logit and take the same LeakyReLU
// decision.  (Forming d_j = <a_dst, m_j> from the feature row that a lane has loaded anyway, instead of
// gathering it, was measured: the butterfly over the head's lanes costs more than the 32-byte gather.)
// Rows cut by a segment boundary are stitched as in the SpMM: inside a block through LDS, across blocks
// through two partials per block and a second kernel; every combination has a fixed order, so results
// are reproducible.
//
// A group walks its segment in batches of two entries with two batches in flight: the gathers of the next
// batch are issued before the current one is folded.  (Loads and stores share one in-order counter on this
// chip; with a single batch in flight every wait for a gather also waited for the stores of the rows just
// completed, and the gather latency itself was exposed once per batch: the forward pass ran a quarter slower.)
// Gathers are addressed as uniform base + 32-bit byte offset, the offset one 24-bit multiply-add; graphs or
// arrays too large for that run the unfused kernels.
#include "common.h"

namespace gnn {
namespace {

__device__ __forceinline__ float leaky(float y, float slope) { return y > 0.f ? y : slope * y; }

// What a lane of a segment group works on.
struct Lane {
    int foff;        // first of its four features (index into a row of f floats)
    int hd;          // head of those features
    bool ok;         // the lane has features (the tile may be narrower than the group)
    bool leader;     // first lane of its head: writes the per-head results
};

struct Geo {
    int h, k, f;         // heads, features per head, f = h k
    int tile_heads;      // heads per feature tile (blockIdx.y picks the tile)
    int lh;              // lanes per head = k / 4
    __device__ Lane lane(int l, int tile) const {
        Lane ln;
        const int in_tile = 4 * l;
        const int hd = tile * tile_heads + in_tile / k;
        ln.ok = in_tile < tile_heads * k && hd < h;
        ln.hd = ln.ok ? hd : 0;
        ln.foff = ln.ok ? tile * tile_heads * k + in_tile : 0;
        ln.leader = ln.ok && (l % lh) == 0;
        return ln;
    }
};

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
// Gathers address their operand as a uniform base plus an unsigned 32-bit byte offset (arrays below 4 GiB), the
// offset one 24-bit multiply-add: index * (bytes per row) + the lane's own part.  Node numbers are below 2^24
// and rows shorter than 2^24 bytes (checked on the host); offsets built from entry slots take a full multiply.
__device__ __forceinline__ uint32_t off24(int idx, uint32_t row_bytes, uint32_t lane_bytes) {
    return __umul24((uint32_t)idx, row_bytes) + lane_bytes;
}
__device__ __forceinline__ uint32_t off32(int idx, uint32_t row_bytes, uint32_t lane_bytes) {
    return (uint32_t)idx * row_bytes + lane_bytes;
}
template <class T> __device__ __forceinline__ T ldb(const void *base, uint32_t byte_off) {
    return *reinterpret_cast<const T *>(static_cast<const char *>(base) + byte_off);
}
// A lane's constant offsets: its four features inside a row of f floats, its head inside rows of h
// floats, h bytes and h float4s.
struct LaneOff {
    uint32_t feat, head4, head1, head16;
};
__device__ __forceinline__ LaneOff lane_off(const Lane &ln) {
    return LaneOff{(uint32_t)ln.foff * 4u, (uint32_t)ln.hd * 4u, (uint32_t)ln.hd, (uint32_t)ln.hd * 16u};
}
__device__ __forceinline__ float dot4(const float4 &a, const float4 &b) {
    return fmaf(a.w, b.w, fmaf(a.z, b.z, fmaf(a.y, b.y, a.x * b.x)));
}
// sum over the lanes of one head (lh consecutive lanes, lh a power of two)
__device__ __forceinline__ float head_sum(float v, int lh) {
    for (int o = lh >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// What a lane accumulates per row: NF floats and ND doubles.  Partials travel through LDS and the partial
// buffers in slots of Acc::WORDS 32-bit words (an even number; the doubles come first, 8-byte aligned).
template <int NF_, int ND_>
struct Acc {
    static constexpr int NF = NF_, ND = ND_, WORDS = (2 * ND_ + NF_ + 1) / 2 * 2;
    float f[NF_ > 0 ? NF_ : 1];
    double d[ND_ > 0 ? ND_ : 1];
    __device__ void store(float *slot) const {
#pragma unroll
        for (int i = 0; i < ND; ++i) reinterpret_cast<double *>(slot)[i] = d[i];
#pragma unroll
        for (int i = 0; i < NF; ++i) slot[2 * ND + i] = f[i];
    }
    __device__ void load(const float *slot) {
#pragma unroll
        for (int i = 0; i < ND; ++i) d[i] = reinterpret_cast<const double *>(slot)[i];
#pragma unroll
        for (int i = 0; i < NF; ++i) f[i] = slot[2 * ND + i];
    }
};

// ---- forward: online softmax + aggregation -------------------------------------------------------
// f = (a0..a3: sum of exp(w - m) M_j over the entries seen, m, l)
struct FwdOp {
    typedef Acc<6, 0> A;
    Geo geo;
    const float *M, *s, *d;
    float slope;
    const float *bias;
    int act;
    float *Y, *stat;
    struct Ent { float4 m; float sv, dv; };
    __device__ void init(A &a) const { a.f[0] = a.f[1] = a.f[2] = a.f[3] = 0.f; a.f[4] = -INFINITY; a.f[5] = 0.f; }
    __device__ void load(Ent &e, int row, int col, int slot, const LaneOff &lo) const {
        (void)slot;
        e.m = ldb<float4>(M, off24(col, geo.f * 4u, lo.feat));
        e.sv = ldb<float>(s, off24(row, geo.h * 4u, lo.head4));
        e.dv = ldb<float>(d, off24(col, geo.h * 4u, lo.head4));
    }
    __device__ void prepare(Ent &, const Lane &) const {}
    __device__ void fold(A &a, const Ent &e) const {
        // one of the two factors exp(m - max), exp(w - max) is exp(0): one exponential of -|w - m| serves both
        const float w = leaky(e.sv + e.dv, slope);
        const float ex = __expf(-fabsf(w - a.f[4]));                 // m = -inf at the start of a row: 0
        const bool grow = w > a.f[4];
        const float sc = grow ? ex : 1.f, p = grow ? 1.f : ex;
        a.f[0] = fmaf(p, e.m.x, a.f[0] * sc); a.f[1] = fmaf(p, e.m.y, a.f[1] * sc);
        a.f[2] = fmaf(p, e.m.z, a.f[2] * sc); a.f[3] = fmaf(p, e.m.w, a.f[3] * sc);
        a.f[5] = fmaf(a.f[5], sc, p);
        a.f[4] = grow ? w : a.f[4];
    }
    __device__ static void combine(A &a, const A &b) {
        if (b.f[4] == -INFINITY) return;                             // b holds no entry
        const float mx = fmaxf(a.f[4], b.f[4]);
        const float sa = __expf(a.f[4] - mx), sb = __expf(b.f[4] - mx);
#pragma unroll
        for (int i = 0; i < 4; ++i) a.f[i] = fmaf(a.f[i], sa, b.f[i] * sb);
        a.f[5] = fmaf(a.f[5], sa, b.f[5] * sb);
        a.f[4] = mx;
    }
    // ELU through exp(x) - 1: its absolute error near zero (one float rounding of a number close to 1) is far
    // below the tolerance of the outputs, and the row finish, instantiated at every entry of the unrolled walk,
    // stays short
    __device__ float epi(float x, int c) const {
        if (bias) x += bias[c];
        if (act == kActRelu) x = fmaxf(x, 0.f);
        else if (act == kActElu) x = x > 0.f ? x : __expf(x) - 1.f;
        return x;
    }
    __device__ void finish(int row, const Lane &ln, const A &a) const {
        if (!ln.ok) return;
        const float inv = __builtin_amdgcn_rcpf(a.f[5]);             // l >= 1: one ulp is far inside the tolerance
        const int c = ln.foff;
        float4 y = make_float4(a.f[0] * inv, a.f[1] * inv, a.f[2] * inv, a.f[3] * inv);
        if (bias) {
            const float4 b = ld4(bias + c);
            y.x += b.x; y.y += b.y; y.z += b.z; y.w += b.w;
        }
        if (act == kActRelu) {
            y.x = fmaxf(y.x, 0.f); y.y = fmaxf(y.y, 0.f); y.z = fmaxf(y.z, 0.f); y.w = fmaxf(y.w, 0.f);
        } else if (act == kActElu) {
            y.x = y.x > 0.f ? y.x : __expf(y.x) - 1.f; y.y = y.y > 0.f ? y.y : __expf(y.y) - 1.f;
            y.z = y.z > 0.f ? y.z : __expf(y.z) - 1.f; y.w = y.w > 0.f ? y.w : __expf(y.w) - 1.f;
        }
        *reinterpret_cast<float4 *>(Y + (size_t)row * geo.f + c) = y;
        if (ln.leader) {
            float *st = stat + ((size_t)row * geo.h + ln.hd) * 2;
            st[0] = a.f[4];
            st[1] = a.f[5];
        }
    }
    // a row without entries aggregates nothing: Y_i = act(b); tile 0 writes it
    __device__ void finish_empty(long row, int tile) const {
        if (tile != 0) return;
        for (int c = 0; c < geo.f; ++c) Y[(size_t)row * geo.f + c] = epi(0.f, c);
        for (int p = 0; p < geo.h; ++p) { stat[((size_t)row * geo.h + p) * 2] = 0.f; stat[((size_t)row * geo.h + p) * 2 + 1] = 1.f; }
    }
};

// ---- backward, row pass: SDDMM folded into the row sums ---------------------------------------------
// The row sums are kept in double: ds = (1 - beta)(P - t Q) cancels almost completely when the softmax of a
// row is concentrated on one entry with a positive logit (P and t Q both approach that entry's g_alpha), and
// the float rounding of three long sums would be what is left.
//
// Cached alpha and mask.  d = (t, P, Q), the same in every lane of a head.
struct BwdRowCachedOp {
    typedef Acc<0, 3> A;
    Geo geo;
    const float *G, *M;
    const float *alpha;       // [q][h]
    const uint8_t *mask;      // [q][h]
    float slope;
    float *ds;                // [n][h]
    float *node;              // t [n][h]
    struct Ent { float4 m, g; float al, pos, ga; };
    __device__ void init(A &a) const { a.d[0] = a.d[1] = a.d[2] = 0.0; }
    __device__ void load(Ent &e, int row, int col, int slot, const LaneOff &lo) const {
        e.m = ldb<float4>(M, off24(col, geo.f * 4u, lo.feat));
        e.g = ldb<float4>(G, off24(row, geo.f * 4u, lo.feat));
        e.al = ldb<float>(alpha, off32(slot, geo.h * 4u, lo.head4));
        e.pos = ldb<uint8_t>(mask, off32(slot, geo.h, lo.head1)) ? 1.f : 0.f;
    }
    __device__ void prepare(Ent &e, const Lane &ln) const { e.ga = head_sum(ln.ok ? dot4(e.m, e.g) : 0.f, geo.lh); }
    __device__ void fold(A &a, const Ent &e) const {
        const double x = (double)e.al * (double)e.ga, pos = (double)e.pos;
        a.d[0] += x;
        a.d[1] += pos * x;
        a.d[2] += pos * (double)e.al;
    }
    __device__ static void combine(A &a, const A &b) { a.d[0] += b.d[0]; a.d[1] += b.d[1]; a.d[2] += b.d[2]; }
    __device__ void finish(int row, const Lane &ln, const A &a) const {
        if (!ln.leader) return;
        const size_t ih = (size_t)row * geo.h + ln.hd;
        ds[ih] = (float)((1.0 - (double)slope) * (a.d[1] - a.d[0] * a.d[2]));
        node[ih] = (float)a.d[0];
    }
    __device__ void finish_empty(long row, int tile) const {
        if (tile != 0) return;
        for (int p = 0; p < geo.h; ++p) { ds[(size_t)row * geo.h + p] = 0.f; node[(size_t)row * geo.h + p] = 0.f; }
    }
};

// alpha rebuilt: f = (m), d = (l, T, P', Q') with l = sum exp(w - m), T = sum exp(w - m) g_alpha, P', Q' the
// same sums over the entries with a positive logit; t = T / l, P = P' / l, Q = Q' / l when the row is
// complete.  Numerator and denominator use the same exponentials, so their rounding cancels in the ratios.
struct BwdRowOnlineOp {
    typedef Acc<1, 4> A;
    Geo geo;
    const float *G, *M, *s, *d;
    float slope;
    float *ds;                // [n][h]
    float *node;              // (s_i, m_i, 1 / l_i, t_i) [n][h][4]
    struct Ent { float4 m, g; float sv, dv, ga; };
    __device__ void init(A &a) const { a.f[0] = -INFINITY; a.d[0] = a.d[1] = a.d[2] = a.d[3] = 0.0; }
    __device__ void load(Ent &e, int row, int col, int slot, const LaneOff &lo) const {
        (void)slot;
        e.m = ldb<float4>(M, off24(col, geo.f * 4u, lo.feat));
        e.g = ldb<float4>(G, off24(row, geo.f * 4u, lo.feat));
        e.sv = ldb<float>(s, off24(row, geo.h * 4u, lo.head4));
        e.dv = ldb<float>(d, off24(col, geo.h * 4u, lo.head4));
    }
    __device__ void prepare(Ent &e, const Lane &ln) const { e.ga = head_sum(ln.ok ? dot4(e.m, e.g) : 0.f, geo.lh); }
    __device__ void fold(A &a, const Ent &e) const {
        const float y = e.sv + e.dv, w = leaky(y, slope);
        const float ex = __expf(-fabsf(w - a.f[0]));                 // as in the forward pass: one exponential
        const bool grow = w > a.f[0];
        const double sc = grow ? (double)ex : 1.0, p = grow ? 1.0 : (double)ex;
        const double pg = p * (double)e.ga, pos = y > 0.f ? 1.0 : 0.0;
        a.d[0] = a.d[0] * sc + p;
        a.d[1] = a.d[1] * sc + pg;
        a.d[2] = a.d[2] * sc + pos * pg;
        a.d[3] = a.d[3] * sc + pos * p;
        a.f[0] = grow ? w : a.f[0];
    }
    __device__ static void combine(A &a, const A &b) {
        if (b.f[0] == -INFINITY) return;
        const float mx = fmaxf(a.f[0], b.f[0]);
        const double sa = (double)__expf(a.f[0] - mx), sb = (double)__expf(b.f[0] - mx);
#pragma unroll
        for (int i = 0; i < 4; ++i) a.d[i] = a.d[i] * sa + b.d[i] * sb;
        a.f[0] = mx;
    }
    __device__ void finish(int row, const Lane &ln, const A &a) const {
        if (!ln.leader) return;
        const size_t ih = (size_t)row * geo.h + ln.hd;
        const double inv = 1.0 / a.d[0];
        const double t = a.d[1] * inv;
        ds[ih] = (float)((1.0 - (double)slope) * (a.d[2] * inv - t * (a.d[3] * inv)));
        *reinterpret_cast<float4 *>(node + ih * 4) = make_float4(s[ih], a.f[0], (float)inv, (float)t);
    }
    __device__ void finish_empty(long row, int tile) const {
        if (tile != 0) return;
        for (int p = 0; p < geo.h; ++p) {
            const size_t ih = (size_t)row * geo.h + p;
            ds[ih] = 0.f;
            *reinterpret_cast<float4 *>(node + ih * 4) = make_float4(0.f, 0.f, 1.f, 0.f);
        }
    }
};

// ---- backward, column pass: dd and dM = A^T G + ds a_src + dd a_dst ----------------------------------
// Here "row" is the column j of the matrix (the pass walks the CSC arrays), "col" the row i of the entry.
// f = (a0..a3: sum alpha_e G_i, dd)
template <bool CACHED>
struct BwdColOp {
    typedef Acc<5, 0> A;
    Geo geo;
    const float *G, *M;
    const float *alpha;            // CACHED: [q][h] and the mask, in CSR order
    const uint8_t *mask;
    const float *node;             // CACHED: t [n][h]; else (s, m, 1 / l, t) [n][h][4], as written by the row pass
    const float *d;                // !CACHED: [n][h]
    float slope;
    const float *ds, *a_src, *a_dst;
    float *dd, *dM;
    struct Ent { float4 g, m, nd; float al, pos, t, dv, ga; };
    __device__ void init(A &a) const { a.f[0] = a.f[1] = a.f[2] = a.f[3] = a.f[4] = 0.f; }
    __device__ void load(Ent &e, int j, int i, int slot, const LaneOff &lo) const {
        e.g = ldb<float4>(G, off24(i, geo.f * 4u, lo.feat));
        e.m = ldb<float4>(M, off24(j, geo.f * 4u, lo.feat));
        if constexpr (CACHED) {
            e.al = ldb<float>(alpha, off32(slot, geo.h * 4u, lo.head4));   // through perm: the slot in CSR order
            e.pos = ldb<uint8_t>(mask, off32(slot, geo.h, lo.head1)) ? 1.f : 0.f;
            e.t = ldb<float>(node, off24(i, geo.h * 4u, lo.head4));
        } else {
            e.nd = ldb<float4>(node, off24(i, geo.h * 16u, lo.head16));     // s_i, m_i, 1 / l_i, t_i
            e.dv = ldb<float>(d, off24(j, geo.h * 4u, lo.head4));
        }
    }
    __device__ void prepare(Ent &e, const Lane &ln) const {
        if constexpr (!CACHED) {
            const float y = e.nd.x + e.dv;                                  // the row pass's logit, bit for bit
            e.pos = y > 0.f ? 1.f : 0.f;
            e.al = __expf(leaky(y, slope) - e.nd.y) * e.nd.z;
            e.t = e.nd.w;
        }
        e.ga = head_sum(ln.ok ? dot4(e.g, e.m) : 0.f, geo.lh);
    }
    __device__ void fold(A &a, const Ent &e) const {
        const float gy = e.al * (e.ga - e.t) * (e.pos != 0.f ? 1.f : slope);
        a.f[4] += gy;
        a.f[0] = fmaf(e.al, e.g.x, a.f[0]); a.f[1] = fmaf(e.al, e.g.y, a.f[1]);
        a.f[2] = fmaf(e.al, e.g.z, a.f[2]); a.f[3] = fmaf(e.al, e.g.w, a.f[3]);
    }
    __device__ static void combine(A &a, const A &b) {
#pragma unroll
        for (int i = 0; i < 5; ++i) a.f[i] += b.f[i];
    }
    __device__ void finish(int j, const Lane &ln, const A &a) const {
        if (!ln.ok) return;
        const size_t jh = (size_t)j * geo.h + ln.hd;
        const float dsv = ds[jh], ddv = a.f[4];
        const float4 u = ld4(a_src + ln.foff), w = ld4(a_dst + ln.foff);           // a_* are [h][k] = [f]
        *reinterpret_cast<float4 *>(dM + (size_t)j * geo.f + ln.foff) =
            make_float4(a.f[0] + dsv * u.x + ddv * w.x, a.f[1] + dsv * u.y + ddv * w.y,
                        a.f[2] + dsv * u.z + ddv * w.z, a.f[3] + dsv * u.w + ddv * w.w);
        if (ln.leader) dd[jh] = ddv;
    }
    // a node that nobody reads: dd_j = 0, dM_j = ds_j a_src
    __device__ void finish_empty(long j, int tile) const {
        if (tile != 0) return;
        for (int c = 0; c < geo.f; ++c) dM[(size_t)j * geo.f + c] = ds[(size_t)j * geo.h + c / geo.k] * a_src[c];
        for (int p = 0; p < geo.h; ++p) dd[(size_t)j * geo.h + p] = 0.f;
    }
};

// U consecutive staged indices (aligned: segments and batches are multiples of U entries)
template <int U> __device__ __forceinline__ void read_indices(const int32_t *p, int (&v)[U]) {
    if constexpr (U == 2) {
        const int2 q = *reinterpret_cast<const int2 *>(p);
        v[0] = q.x; v[1] = q.y;
    } else {
#pragma unroll
        for (int u = 0; u < U; u += 4) {
            const int4 q = *reinterpret_cast<const int4 *>(p + u);
            v[u] = q.x; v[u + 1] = q.y; v[u + 2] = q.z; v[u + 3] = q.w;
        }
    }
}

struct WalkInfo {
    int32_t tail_row;      // row whose tail partial this segment holds, or -1
    int32_t has_head;      // the segment's first row began before it
    int32_t whole;         // ... and also continues after it
    int32_t active;        // the segment exists
};

constexpr int kMaxAccWords = 10;       // the widest accumulator (Acc<1, 4>), for sizing the partial buffer

// One group of LPE lanes per segment of `seg` entries, GPB = 256 / LPE groups per block.  rowidx / colidx:
// row and column of every entry in walking order; slotidx: its slot in the per-edge arrays (NULL: the
// walking order itself).  Partials of rows that cross the block's span go to part[tile][2 b (+1)][LPE][words].
template <class Op, int LPE, int U>
__global__ void __launch_bounds__(256)
seg_walk_kernel(int nnz, int seg, long nseg, const int32_t *__restrict__ rowidx, const int32_t *__restrict__ colidx,
                const int32_t *__restrict__ slotidx, Op op, float *__restrict__ part) {
    extern __shared__ __align__(16) int32_t smem[];
    typedef typename Op::A A;
    constexpr int GPB = 256 / LPE, W = A::WORDS;
    static_assert(W <= kMaxAccWords, "partial buffer too small");
    const int span = GPB * seg;                                           // a multiple of 4: the floats below stay aligned
    int32_t *s_row = smem, *s_col = smem + span, *s_slot = smem + 2 * span;
    float *s_head = reinterpret_cast<float *>(smem + 3 * span);          // [GPB][LPE][W]
    float *s_tail = s_head + 256 * W;
    WalkInfo *s_info = reinterpret_cast<WalkInfo *>(s_tail + 256 * W);
    const long blk_first = (long)blockIdx.x * span;
    for (int i = threadIdx.x; i < span; i += 256) {
        const long x = blk_first + i;
        const bool in = x < nnz;                           // past the end: entry 0 of row / column 0, loaded but never folded
        s_row[i] = in ? rowidx[x] : 0;
        s_col[i] = in ? colidx[x] : 0;
        s_slot[i] = in ? (slotidx ? slotidx[x] : (int)x) : 0;
    }
    __syncthreads();
    const int l = threadIdx.x % LPE, gl = threadIdx.x / LPE;
    const long g = (long)blockIdx.x * GPB + gl;
    const bool active = g < nseg;
    const Lane ln = op.geo.lane(l, blockIdx.y);
    const LaneOff lo = lane_off(ln);
    float *part_tile = part + (size_t)blockIdx.y * 2 * gridDim.x * (LPE * W);
    A acc;
    op.init(acc);
    float *my_head = s_head + (gl * LPE + l) * W, *my_tail = s_tail + (gl * LPE + l) * W;
    WalkInfo info{-1, 0, 0, active ? 1 : 0};
    if (active) {
        const int lb = gl * seg;
        const long s0 = g * seg;
        const int cnt = (int)min((long)seg, (long)nnz - s0);
        const int first = s_row[lb];
        const int before = gl > 0 ? s_row[lb - 1] : (s0 > 0 ? rowidx[s0 - 1] : -1);
        const bool head_open = before == first;
        int cur = first;
        // The segment in batches of U entries, two batches in flight: the gathers of batch b + 1 are issued
        // before batch b is folded, so they (and the stores of the rows that batch b completes) have a whole
        // batch of arithmetic to finish in.  seg is a multiple of 2 U; every batch of the segment is loaded,
        // also past the entry list's end (the staged filler: entry 0 of row 0, loaded and not folded), and
        // the batch after the last one is the last one again.
        typedef typename Op::Ent Ent;
        auto fetch = [&](int x, int (&r)[U], Ent (&ent)[U]) __attribute__((always_inline)) {
            int c[U], sl[U];
            read_indices<U>(s_row + lb + x, r);
            read_indices<U>(s_col + lb + x, c);
            read_indices<U>(s_slot + lb + x, sl);
#pragma unroll
            for (int u = 0; u < U; ++u) op.load(ent[u], r[u], c[u], sl[u], lo);       // lanes without features read feature 0
        };
        auto consume = [&](int x, const int (&r)[U], Ent (&ent)[U]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < U; ++u) op.prepare(ent[u], ln);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (x + u < cnt) {
                    if (r[u] != cur) {
                        if (cur == first && head_open) acc.store(my_head);
                        else op.finish(cur, ln, acc);
                        op.init(acc);
                        cur = r[u];
                    }
                    op.fold(acc, ent[u]);
                }
            }
        };
        int ra[U], rb[U];
        Ent ea[U], eb[U];
        fetch(0, ra, ea);
        for (int x = 0; x < seg; x += 2 * U) {
            fetch(x + U, rb, eb);
            consume(x, ra, ea);
            fetch(x + 2 * U < seg ? x + 2 * U : seg - U, ra, ea);
            consume(x + U, rb, eb);
        }
        const long e = s0 + cnt;
        const int after = e >= nnz ? -1 : (gl + 1 < GPB ? s_row[lb + seg] : rowidx[e]);
        const bool in_head = cur == first && head_open;
        info.has_head = head_open ? 1 : 0;
        if (in_head) {
            acc.store(my_head);
            info.whole = after == cur ? 1 : 0;
        } else if (after == cur) {
            acc.store(my_tail);
            info.tail_row = cur;
        } else {
            op.finish(cur, ln, acc);
        }
    }
    if (l == 0) s_info[gl] = info;
    __syncthreads();
    if (!active) return;

    A b;
    if (info.tail_row >= 0) {                  // add the heads of the following segments of the block, in order
        acc.load(my_tail);
        bool open = true;
        for (int x = gl + 1; x < GPB && s_info[x].active; ++x) {
            b.load(s_head + (x * LPE + l) * W);
            Op::combine(acc, b);
            if (!s_info[x].whole) { open = false; break; }
        }
        if (open) acc.store(part_tile + ((size_t)(2 * blockIdx.x + 1) * LPE + l) * W);   // continues past the block
        else op.finish(info.tail_row, ln, acc);
    }
    if (gl == 0 && info.has_head) {            // the row that began before the block
        acc.load(s_head + l * W);
        for (int x = 0; s_info[x].whole && x + 1 < GPB && s_info[x + 1].active; ++x) {
            b.load(s_head + ((x + 1) * LPE + l) * W);
            Op::combine(acc, b);
        }
        acc.store(part_tile + ((size_t)(2 * blockIdx.x) * LPE + l) * W);
    }
}

// Second kernel, one wavefront per block span b of the first (and per feature tile): if a row starts in span
// b and continues past its end, combine its partials - slot 2b+1, then slot 2x of every later span x it
// reaches - and finish the row.  The 64 lanes form 64 / LPE slots; slot s takes spans b+1+s, b+1+s+slots, ...
// in order, the slots are combined by a fixed xor tree.  Lane i of wavefront w also finishes row 64 w + i
// if it has no entry at all.
template <class Op, int LPE>
__global__ void __launch_bounds__(256)
seg_fixup_kernel(int n, int nnz, int span, long nspan, const int32_t *__restrict__ rowidx,
                 const int32_t *__restrict__ ptr, Op op, const float *__restrict__ part) {
    typedef typename Op::A A;
    constexpr int W = A::WORDS, SLOTS = kWave / LPE;
    const int lane = threadIdx.x % kWave;
    const long g = (long)blockIdx.x * 4 + threadIdx.x / kWave;
    const long row = g * kWave + lane;
    if (row < n && ptr[row] == ptr[row + 1]) op.finish_empty(row, blockIdx.y);
    if (g >= nspan) return;
    const long e = (g + 1) * span;
    if (e >= nnz) return;                                  // nothing follows the last span
    const int r = rowidx[e - 1];
    if (rowidx[e] != r) return;                            // the boundary falls between two rows
    const long s0 = g * span;
    if (s0 > 0 && rowidx[s0 - 1] == r) return;             // the row began earlier: its first span owns it
    const long g_end = ((long)ptr[r + 1] - 1) / span;
    const int l = lane % LPE, slot = lane / LPE;
    const Lane ln = op.geo.lane(l, blockIdx.y);
    const float *part_tile = part + (size_t)blockIdx.y * 2 * nspan * (LPE * W);
    A acc, b;
    op.init(acc);
    for (long x = g + 1 + slot; x <= g_end; x += SLOTS) {
        b.load(part_tile + ((size_t)(2 * x) * LPE + l) * W);
        Op::combine(acc, b);
    }
    for (int d = LPE; d < kWave; d <<= 1) {
#pragma unroll
        for (int i = 0; i < A::NF; ++i) b.f[i] = __shfl_xor(acc.f[i], d, kWave);
#pragma unroll
        for (int i = 0; i < A::ND; ++i) b.d[i] = __shfl_xor(acc.d[i], d, kWave);
        Op::combine(acc, b);
    }
    if (slot == 0) {
        A t;
        t.load(part_tile + ((size_t)(2 * g + 1) * LPE + l) * W);
        Op::combine(t, acc);
        op.finish(r, ln, t);
    }
}

int pow2_at_least(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

struct Shape {
    Geo geo;
    int lpe, tiles, seg;
    long nseg, nblk;
};

Shape pick_shape(int64_t nnz, int h, int k) {
    Shape sh;
    sh.geo.h = h; sh.geo.k = k; sh.geo.f = h * k;
    sh.geo.lh = k / 4;
    sh.geo.tile_heads = h * k <= 256 ? h : (256 / k);
    sh.tiles = (h + sh.geo.tile_heads - 1) / sh.geo.tile_heads;
    sh.lpe = pow2_at_least(sh.geo.tile_heads * k / 4);
    if (sh.lpe < 2) sh.lpe = 2;
    // as long as possible while the chip still gets about eight wavefronts per SIMD; index staging <= 24 KB
    const int64_t want_groups = (int64_t)8192 * (kWave / sh.lpe) / sh.tiles;
    const int64_t want = nnz / (want_groups > 0 ? want_groups : 1);
    const int cap = 8 * sh.lpe < 256 ? 8 * sh.lpe : 256;
    sh.seg = 16;
    while (sh.seg * 2 <= want && sh.seg * 2 <= cap) sh.seg <<= 1;
    sh.nseg = ceil_div(nnz, sh.seg);
    sh.nblk = ceil_div(sh.nseg, 256 / sh.lpe);
    return sh;
}

template <class Op, int U>
gnn_status_t run_pass(const Shape &sh, int n, int nnz, const int32_t *ptr, const int32_t *rowidx,
                      const int32_t *colidx, const int32_t *slotidx, Op op, float *part, hipStream_t st) {
    op.geo = sh.geo;
    const int gpb = 256 / sh.lpe, span = gpb * sh.seg;
    const size_t lds = (size_t)3 * span * sizeof(int32_t) + (size_t)2 * 256 * Op::A::WORDS * sizeof(float) +
                       (size_t)gpb * sizeof(WalkInfo);
    const dim3 grid((unsigned)sh.nblk, (unsigned)sh.tiles);
    const long waves = sh.nblk > ceil_div(n, kWave) ? sh.nblk : ceil_div(n, kWave);
    const dim3 fgrid((unsigned)ceil_div(waves, 4), (unsigned)sh.tiles);
#define PASS_CASE(LPE_)                                                                                           \
    if (sh.lpe == LPE_) {                                                                                         \
        hipLaunchKernelGGL((seg_walk_kernel<Op, LPE_, U>), grid, dim3(256), lds, st, nnz, sh.seg, sh.nseg, rowidx, \
                           colidx, slotidx, op, part);                                                            \
        GNN_TRY(launch_status());                                                                                 \
        hipLaunchKernelGGL((seg_fixup_kernel<Op, LPE_>), fgrid, dim3(256), 0, st, n, nnz, span, sh.nblk, rowidx,  \
                           ptr, op, part);                                                                        \
    }
    PASS_CASE(2) PASS_CASE(4) PASS_CASE(8) PASS_CASE(16) PASS_CASE(32) PASS_CASE(64)
#undef PASS_CASE
    return launch_status();
}

}  // namespace

// The fused passes take feature vectors of whole float4s per head, a power-of-two number of them, and at
// most 256 features per head; other shapes run the unfused kernels.
static bool fused_head_shape(int h, int k) {
    if (h < 1 || k < 4 || k % 4 != 0 || k > 256) return false;
    const int lh = k / 4;
    return (lh & (lh - 1)) == 0;
}

// ... on graphs whose gathers can be addressed with 32-bit byte offsets built by 24-bit multiplies: node
// numbers below 2^24, rows below 2^24 bytes, every gathered array (n x h k floats, n x h float4s, q x h
// floats) below 4 GiB.
bool gat_fused_shape(int64_t n, int64_t nnz, int h, int k) {
    if (!fused_head_shape(h, k)) return false;
    const int64_t f = (int64_t)h * k, lim = (int64_t)1 << 32;
    return n < (1 << 24) && f * 4 < (1 << 24) && n * f * 4 < lim && n * h * 16 < lim && nnz * h * 4 < lim;
}

size_t gat_fused_workspace_bytes(int64_t nnz, int h, int k) {
    if (nnz <= 0 || !fused_head_shape(h, k)) return kAlign;
    const Shape sh = pick_shape(nnz, h, k);
    return align_up((size_t)2 * sh.nblk * sh.tiles * sh.lpe * kMaxAccWords * sizeof(float));
}

gnn_status_t gat_fused_forward_launch(int n, int nnz, int h, int k, const int32_t *rowptr, const int32_t *erow,
                                      const int32_t *col, const float *M, const float *s, const float *d,
                                      float slope, const float *bias, int act, float *Y, float *stat, void *workspace,
                                      hipStream_t st) {
    if (n <= 0) return GNN_OK;
    const Shape sh = pick_shape(nnz > 0 ? nnz : 1, h, k);
    FwdOp op{sh.geo, M, s, d, slope, bias, act, Y, stat};
    if (nnz <= 0) {                                        // every row is empty: the second kernel writes them all
        const dim3 fgrid((unsigned)ceil_div(ceil_div(n, kWave), 4), 1);
        hipLaunchKernelGGL((seg_fixup_kernel<FwdOp, 16>), fgrid, dim3(256), 0, st, n, 0, 1, 0L, erow, rowptr, op,
                           static_cast<const float *>(workspace));
        return launch_status();
    }
    return run_pass<FwdOp, 2>(sh, n, nnz, rowptr, erow, col, nullptr, op, static_cast<float *>(workspace), st);
}

// Row pass (CSR arrays) then column pass (CSC arrays) of the backward edge phase.
//   alpha, mask [q][h] in CSR entry order, or NULL: alpha is rebuilt from s, d [n][h];  node: scratch of 4 n h floats; ds, dd [n][h];
//   dM [n][h k] (complete: rank-one terms included)
gnn_status_t gat_fused_backward_launch(int n, int nnz, int h, int k, const int32_t *rowptr, const int32_t *erow,
                                       const int32_t *col, const int32_t *colptr, const int32_t *ecol,
                                       const int32_t *row, const int32_t *perm, const float *G, const float *M,
                                       const float *alpha, const uint8_t *mask, const float *s,
                                       const float *d, float slope, const float *a_src, const float *a_dst,
                                       float *node, float *ds, float *dd, float *dM, void *workspace, hipStream_t st) {
    if (n <= 0) return GNN_OK;
    const Shape sh = pick_shape(nnz > 0 ? nnz : 1, h, k);
    float *part = static_cast<float *>(workspace);
    if (nnz <= 0) {
        const dim3 fgrid((unsigned)ceil_div(ceil_div(n, kWave), 4), 1);
        BwdRowCachedOp ra{sh.geo, G, M, alpha, mask, slope, ds, node};
        hipLaunchKernelGGL((seg_fixup_kernel<BwdRowCachedOp, 16>), fgrid, dim3(256), 0, st, n, 0, 1, 0L, erow, rowptr, ra, part);
        GNN_TRY(launch_status());
        BwdColOp<true> cb{sh.geo, G, M, alpha, mask, node, nullptr, slope, ds, a_src, a_dst, dd, dM};
        hipLaunchKernelGGL((seg_fixup_kernel<BwdColOp<true>, 16>), fgrid, dim3(256), 0, st, n, 0, 1, 0L, ecol, colptr, cb, part);
        return launch_status();
    }
    if (alpha) {
        BwdRowCachedOp ra{sh.geo, G, M, alpha, mask, slope, ds, node};
        GNN_TRY((run_pass<BwdRowCachedOp, 2>(sh, n, nnz, rowptr, erow, col, nullptr, ra, part, st)));
        BwdColOp<true> cb{sh.geo, G, M, alpha, mask, node, nullptr, slope, ds, a_src, a_dst, dd, dM};
        return run_pass<BwdColOp<true>, 2>(sh, n, nnz, colptr, ecol, row, perm, cb, part, st);
    }
    BwdRowOnlineOp ra{sh.geo, G, M, s, d, slope, ds, node};
    GNN_TRY((run_pass<BwdRowOnlineOp, 2>(sh, n, nnz, rowptr, erow, col, nullptr, ra, part, st)));
    BwdColOp<false> cb{sh.geo, G, M, nullptr, nullptr, node, d, slope, ds, a_src, a_dst, dd, dM};
    return run_pass<BwdColOp<false>, 2>(sh, n, nnz, colptr, ecol, row, perm, cb, part, st);
}

}  // namespace gnn
