// GAT kernels (Sec. "GAT Forward Pass", "GAT Backward Pass", App. B) for gfx950.
//
// All per-edge tensors are [nnz][heads] and all per-node tensors [n][heads] or
// [n][heads][dim]: the head is the last / middle axis, so the `heads` values of one
// edge or node sit in one cache line and are handled by neighbouring lanes (Sec. 3.2).
//
// Two kernel shapes cover every step:
//   * entry-parallel kernels, one thread per (entry, head): logits -> alpha, the SDDMM
//     dot products, the chain rule through softmax and LeakyReLU.  They need the row
//     of each entry, hence the expanded row index `erow`.
//   * an entry-balanced row reduction (head_walker_kernel): like the SpMM it cuts the
//     entry list into equal segments, one group of lanes (one lane per head) per
//     segment, keeps a running reduction per row and leaves partials for rows that a
//     segment boundary cuts; a second kernel combines the partials in segment order.
//     It computes the softmax statistics (running max and sum of exponentials) and
//     the three row sums the backward pass needs.
#include "common.h"

namespace gnn {
namespace {

__device__ __forceinline__ float leaky(float y, float slope) { return y > 0.f ? y : slope * y; }

// ---- s_i = <a_src, m_i>, d_i = <a_dst, m_i> per head (App. B) ------------------------
// VEC = 1: one thread per (node, head).  VEC = 4: L lanes per (node, head), lane l takes the float4 chunks
// l, l + L, ... of the k features (L * 4 <= k, so a wavefront reads consecutive memory), partial dot
// products are combined by a fixed xor tree.
template <int VEC, int L>
__global__ void __launch_bounds__(256)
node_attention_kernel(long count, int h, int k, const float *__restrict__ M, const float *__restrict__ a_src,
                      const float *__restrict__ a_dst, float *__restrict__ s, float *__restrict__ d) {
    const long t = ((long)blockIdx.x * 256 + threadIdx.x) / L;      // t = i * h + p
    const int l = threadIdx.x % L;
    const bool live = t < count;
    float ss = 0.f, dd = 0.f;
    if (live) {
        const int p = count < (1L << 31) ? (int)((unsigned)t % (unsigned)h) : (int)(t % h);
        const float *m = M + (size_t)t * k;
        const float *as = a_src + (size_t)p * k, *ad = a_dst + (size_t)p * k;
        if constexpr (VEC == 4) {
            for (int c = 4 * l; c < k; c += 4 * L) {
                const float4 v = *reinterpret_cast<const float4 *>(m + c);
                const float4 u = *reinterpret_cast<const float4 *>(as + c), w = *reinterpret_cast<const float4 *>(ad + c);
                ss = fmaf(u.x, v.x, ss); ss = fmaf(u.y, v.y, ss); ss = fmaf(u.z, v.z, ss); ss = fmaf(u.w, v.w, ss);
                dd = fmaf(w.x, v.x, dd); dd = fmaf(w.y, v.y, dd); dd = fmaf(w.z, v.z, dd); dd = fmaf(w.w, v.w, dd);
            }
        } else {
            for (int c = 0; c < k; ++c) {
                const float v = m[c];
                ss = fmaf(as[c], v, ss);
                dd = fmaf(ad[c], v, dd);
            }
        }
    }
#pragma unroll
    for (int o = L >> 1; o > 0; o >>= 1) {
        ss += __shfl_xor(ss, o);
        dd += __shfl_xor(dd, o);
    }
    if (live && l == 0) {
        s[t] = ss;
        d[t] = dd;
    }
}

// ---- entry-balanced reduction over the rows, one lane per head -----------------------
// Op::NACC floats per (row, head).  Softmax statistics keep (max, sum of exp(w - max)).
struct StatsOp {
    static constexpr int NACC = 2;
    const float *s, *d;
    float slope;
    __device__ void init(float (&a)[2]) const { a[0] = -INFINITY; a[1] = 0.f; }
    __device__ void load(long e, int r, int c, int h, int p, float (&v)[3]) const {
        (void)e;
        v[0] = s[(size_t)r * h + p];
        v[1] = d[(size_t)c * h + p];
    }
    __device__ void fold(float (&a)[2], const float (&v)[3]) const {
        const float w = leaky(v[0] + v[1], slope);
        if (w > a[0]) { a[1] = a[1] * __expf(a[0] - w) + 1.f; a[0] = w; }
        else a[1] += __expf(w - a[0]);
    }
    __device__ static void combine(float (&a)[2], const float (&b)[2]) {
        if (b[0] == -INFINITY) return;
        const float m = fmaxf(a[0], b[0]);
        a[1] = a[1] * __expf(a[0] - m) + b[1] * __expf(b[0] - m);
        a[0] = m;
    }
};

// Row sums for the backward pass: t = sum alpha*ga, P = sum over y>0 of alpha*ga, Q = sum over y>0 of alpha.
struct SumsOp {
    static constexpr int NACC = 3;
    const float *alpha, *ga;
    const uint8_t *mask;          // NULL: the sign is recomputed from s, d
    const float *s, *d;
    __device__ void init(float (&a)[3]) const { a[0] = a[1] = a[2] = 0.f; }
    __device__ void load(long e, int r, int c, int h, int p, float (&v)[3]) const {
        v[0] = alpha[(size_t)e * h + p];
        v[1] = ga[(size_t)e * h + p];
        if (mask) v[2] = mask[(size_t)e * h + p] ? 1.f : 0.f;
        else v[2] = (s[(size_t)r * h + p] + d[(size_t)c * h + p]) > 0.f ? 1.f : 0.f;
    }
    __device__ void fold(float (&a)[3], const float (&v)[3]) const {
        const float x = v[0] * v[1];
        a[0] += x;
        a[1] += v[2] * x;
        a[2] += v[2] * v[0];
    }
    __device__ static void combine(float (&a)[3], const float (&b)[3]) {
        a[0] += b[0]; a[1] += b[1]; a[2] += b[2];
    }
};

struct WalkInfo {
    int32_t tail_row;      // row whose tail partial this segment holds, or -1
    int32_t has_head;      // the segment's first row began before it
    int32_t whole;         // ... and also continues after it
    int32_t active;        // the segment exists
};

// One group of HP lanes (lane = head) per segment of `seg` entries, GPB groups per block.
// Rows inside a segment are written directly; rows cut by a segment boundary inside the
// block are stitched through LDS after a barrier (the group holding the tail of a row
// combines the heads of the following segments in order); only rows that cross the block's
// span leave partials in global memory (slot 2b: began before block b, slot 2b+1: continues
// after it) for head_fixup_kernel.
template <class Op, int HP, int U>
__global__ void __launch_bounds__(256)
head_walker_kernel(int nnz, int h, int seg, long nseg, const int32_t *__restrict__ erow,
                   const int32_t *__restrict__ col, Op op, float *__restrict__ out, float *__restrict__ part) {
    extern __shared__ __align__(16) int32_t smem[];
    constexpr int GPB = 256 / HP, NA = Op::NACC;
    const int span = GPB * seg;
    int32_t *s_row = smem, *s_col = smem + span;
    float *s_head = reinterpret_cast<float *>(smem + 2 * span);        // [GPB][HP][NA]
    float *s_tail = s_head + GPB * HP * NA;
    WalkInfo *s_info = reinterpret_cast<WalkInfo *>(s_tail + GPB * HP * NA);
    const long blk_first = (long)blockIdx.x * span;
    for (int i = threadIdx.x; i < span; i += 256) {
        const long x = blk_first + i;
        if (x < nnz) { s_row[i] = erow[x]; s_col[i] = col[x]; }
    }
    __syncthreads();
    const int p = threadIdx.x % HP, gl = threadIdx.x / HP;
    const long g = (long)blockIdx.x * GPB + gl;
    const bool active = g < nseg;
    const bool lane_on = p < h;
    float acc[NA];
    op.init(acc);
    float *my_head = s_head + (gl * HP + p) * NA, *my_tail = s_tail + (gl * HP + p) * NA;
    WalkInfo info{-1, 0, 0, active ? 1 : 0};
    if (active) {
        const int lb = gl * seg;
        const long s0 = g * seg;
        const int cnt = (int)min((long)seg, (long)nnz - s0);
        const int first = s_row[lb];
        const int before = gl > 0 ? s_row[lb - 1] : (s0 > 0 ? erow[s0 - 1] : -1);
        const bool head_open = before == first;
        int cur = first;
        for (int x = 0; x < cnt; x += U) {
            int r[U], c[U];
            float v[U][3];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = lb + min(x + u, cnt - 1);
                r[u] = s_row[i];
                c[u] = s_col[i];
            }
            if (lane_on) {
#pragma unroll
                for (int u = 0; u < U; ++u) op.load(s0 + min(x + u, cnt - 1), r[u], c[u], h, p, v[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (x + u < cnt) {
                    if (r[u] != cur) {
                        if (lane_on) {
                            float *dst = (cur == first && head_open) ? my_head : out + ((size_t)cur * h + p) * NA;
#pragma unroll
                            for (int a = 0; a < NA; ++a) dst[a] = acc[a];
                        }
                        op.init(acc);
                        cur = r[u];
                    }
                    if (lane_on) op.fold(acc, v[u]);
                }
            }
        }
        const long e = s0 + cnt;
        const int after = e >= nnz ? -1 : (gl + 1 < GPB ? s_row[lb + seg] : erow[e]);
        const bool in_head = cur == first && head_open;
        info.has_head = head_open ? 1 : 0;
        float *dst;
        if (in_head) { dst = my_head; info.whole = after == cur ? 1 : 0; }
        else if (after == cur) { dst = my_tail; info.tail_row = cur; }
        else dst = out + ((size_t)cur * h + p) * NA;
        if (lane_on) {
#pragma unroll
            for (int a = 0; a < NA; ++a) dst[a] = acc[a];
        }
    }
    if (p == 0) s_info[gl] = info;
    __syncthreads();
    if (!active || !lane_on) return;

    float b[NA];
    if (info.tail_row >= 0) {
#pragma unroll
        for (int a = 0; a < NA; ++a) acc[a] = my_tail[a];
        bool open = true;
        for (int x = gl + 1; x < GPB && s_info[x].active; ++x) {
#pragma unroll
            for (int a = 0; a < NA; ++a) b[a] = s_head[(x * HP + p) * NA + a];
            Op::combine(acc, b);
            if (!s_info[x].whole) { open = false; break; }
        }
        float *dst = open ? part + (((size_t)(2 * blockIdx.x + 1)) * h + p) * NA
                          : out + ((size_t)info.tail_row * h + p) * NA;
#pragma unroll
        for (int a = 0; a < NA; ++a) dst[a] = acc[a];
    }
    if (gl == 0 && info.has_head) {
#pragma unroll
        for (int a = 0; a < NA; ++a) acc[a] = s_head[p * NA + a];
        for (int x = 0; s_info[x].whole && x + 1 < GPB && s_info[x + 1].active; ++x) {
#pragma unroll
            for (int a = 0; a < NA; ++a) b[a] = s_head[((x + 1) * HP + p) * NA + a];
            Op::combine(acc, b);
        }
        float *dst = part + (((size_t)(2 * blockIdx.x)) * h + p) * NA;
#pragma unroll
        for (int a = 0; a < NA; ++a) dst[a] = acc[a];
    }
}

// Combines the partials of every row that crosses a block span of the walker, one
// wavefront per span b: the 64 lanes form 64 / HP slots of HP lanes (lane = head); slot s
// combines the partials of spans b+1+s, b+1+s+slots, ... in order, the slots are then
// combined by a fixed shuffle tree, and the result joins the tail partial of span b.
template <class Op, int HP>
__global__ void __launch_bounds__(256)
head_fixup_kernel(int nnz, int h, int span, long nspan, const int32_t *__restrict__ erow,
                  const int32_t *__restrict__ rowptr, const float *__restrict__ part, float *__restrict__ out) {
    constexpr int NA = Op::NACC, SLOTS = kWave / HP;
    const int lane = threadIdx.x % kWave;
    const long g = (long)blockIdx.x * 4 + threadIdx.x / kWave;
    if (g >= nspan) return;
    const long e = (g + 1) * span;
    if (e >= nnz) return;
    const int r = erow[e - 1];
    if (erow[e] != r) return;
    const long s0 = g * span;
    if (s0 > 0 && erow[s0 - 1] == r) return;
    const long g_end = ((long)rowptr[r + 1] - 1) / span;
    const int p = lane % HP, slot = lane / HP;
    const bool lane_on = p < h;
    Op op{};
    float acc[NA], b[NA];
    op.init(acc);
    if (lane_on)
        for (long x = g + 1 + slot; x <= g_end; x += SLOTS) {
            const float *src = part + (((size_t)(2 * x)) * h + p) * NA;
#pragma unroll
            for (int a = 0; a < NA; ++a) b[a] = src[a];
            Op::combine(acc, b);
        }
    for (int d = HP; d < kWave; d <<= 1) {
#pragma unroll
        for (int a = 0; a < NA; ++a) b[a] = __shfl_xor(acc[a], d, kWave);
        Op::combine(acc, b);
    }
    if (lane_on && slot == 0) {
        const float *src = part + (((size_t)(2 * g + 1)) * h + p) * NA;
        float t[NA];
#pragma unroll
        for (int a = 0; a < NA; ++a) t[a] = src[a];
        Op::combine(t, acc);
        float *dst = out + ((size_t)r * h + p) * NA;
#pragma unroll
        for (int a = 0; a < NA; ++a) dst[a] = t[a];
    }
}

// ---- entry-parallel kernels ------------------------------------------------------------
// Thread t = e * (h / HV) + pg handles HV consecutive heads of entry e (HV = 4 when h is a
// multiple of 4: every access is then a 16-byte one; the buffers are 256-byte aligned blocks).
__device__ __forceinline__ void split_index(long t, long count, int groups, long &e, int &pg) {
    if (count < (1L << 31)) {                                  // 32-bit division when it is enough
        const unsigned q = (unsigned)t / (unsigned)groups;
        e = q;
        pg = (int)((unsigned)t - q * (unsigned)groups);
    } else {
        e = t / groups;
        pg = (int)(t % groups);
    }
}

template <int HV> __device__ __forceinline__ void load_vec(const float *p, float (&v)[HV]) {
    if constexpr (HV == 4) {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else v[0] = *p;
}
template <int HV> __device__ __forceinline__ void store_vec(float *p, const float (&v)[HV]) {
    if constexpr (HV == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else *p = v[0];
}

// alpha_e = exp(w_e - max_i) / sum_i, mask_e = (y_e > 0)
template <int HV>
__global__ void __launch_bounds__(256)
edge_alpha_kernel(long count, int h, const int32_t *__restrict__ erow, const int32_t *__restrict__ col,
                  const float *__restrict__ s, const float *__restrict__ d, const float *__restrict__ stat,
                  float slope, float *__restrict__ alpha, uint8_t *__restrict__ mask) {
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    long e; int pg;
    split_index(t, count, h / HV, e, pg);
    const int p0 = pg * HV;
    const int r = erow[e], c = col[e];
    float sv[HV], dv[HV], st0[HV], st1[HV], out[HV];
    load_vec<HV>(s + (size_t)r * h + p0, sv);
    load_vec<HV>(d + (size_t)c * h + p0, dv);
    const float *sp = stat + ((size_t)r * h + p0) * 2;            // (max, sum) pairs
    if constexpr (HV == 4) {
        const float4 x = *reinterpret_cast<const float4 *>(sp), y = *reinterpret_cast<const float4 *>(sp + 4);
        st0[0] = x.x; st1[0] = x.y; st0[1] = x.z; st1[1] = x.w; st0[2] = y.x; st1[2] = y.y; st0[3] = y.z; st1[3] = y.w;
    } else { st0[0] = sp[0]; st1[0] = sp[1]; }
    uint8_t m[HV];
#pragma unroll
    for (int i = 0; i < HV; ++i) {
        const float y = sv[i] + dv[i];
        out[i] = __expf(leaky(y, slope) - st0[i]) / st1[i];
        m[i] = y > 0.f;
    }
    store_vec<HV>(alpha + (size_t)e * h + p0, out);
    if (mask) {
        if constexpr (HV == 4) *reinterpret_cast<uchar4 *>(mask + (size_t)e * h + p0) = make_uchar4(m[0], m[1], m[2], m[3]);
        else mask[(size_t)e * h + p0] = m[0];
    }
}

// D_e = val_e * <B_i, Ct_j> per head (App. E.2)
__global__ void __launch_bounds__(256)
sddmm_edge_kernel(long count, int h, int k, const int32_t *__restrict__ erow, const int32_t *__restrict__ col,
                  const float *__restrict__ val, const float *__restrict__ Bm, const float *__restrict__ Ct,
                  float *__restrict__ D, int vec) {
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    const long e = t / h;
    const int p = (int)(t % h);
    const float *b = Bm + ((size_t)erow[e] * h + p) * k;
    const float *c = Ct + ((size_t)col[e] * h + p) * k;
    float acc = 0.f;
    if (vec) {
        for (int x = 0; x < k; x += 4) {
            const float4 u = *reinterpret_cast<const float4 *>(b + x), v = *reinterpret_cast<const float4 *>(c + x);
            acc = fmaf(u.x, v.x, acc); acc = fmaf(u.y, v.y, acc); acc = fmaf(u.z, v.z, acc); acc = fmaf(u.w, v.w, acc);
        }
    } else {
        for (int x = 0; x < k; ++x) acc = fmaf(b[x], c[x], acc);
    }
    D[t] = val ? val[e] * acc : acc;
}

// The same product for long feature vectors (k >= 32, a multiple of 4): L lanes share one (entry, head)
// pair, each reading 16 consecutive bytes per pass, so a pair's two rows are read as whole lines;
// the L partial dot products are added by a fixed butterfly.
template <int L>
__global__ void __launch_bounds__(256)
sddmm_coop_kernel(long pairs, int h, int k, const int32_t *__restrict__ erow, const int32_t *__restrict__ col,
                  const float *__restrict__ val, const float *__restrict__ Bm, const float *__restrict__ Ct,
                  float *__restrict__ D) {
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    const long pair = t / L;
    const int l = (int)(t % L);
    const bool live = pair < pairs;                           // whole groups of L lanes are live or not
    float acc = 0.f;
    long e = 0;
    if (live) {
        int p;
        split_index(pair, pairs, h, e, p);
        const float *b = Bm + ((size_t)erow[e] * h + p) * k;
        const float *c = Ct + ((size_t)col[e] * h + p) * k;
        for (int x = 4 * l; x < k; x += 4 * L) {
            const float4 u = *reinterpret_cast<const float4 *>(b + x), v = *reinterpret_cast<const float4 *>(c + x);
            acc = fmaf(u.x, v.x, acc); acc = fmaf(u.y, v.y, acc); acc = fmaf(u.z, v.z, acc); acc = fmaf(u.w, v.w, acc);
        }
    }
#pragma unroll
    for (int d = L / 2; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, kWave);
    if (live && l == 0) D[pair] = val ? val[e] * acc : acc;
}

// g_y_e = alpha_e (g_alpha_e - t_i) * (y_e > 0 ? 1 : beta); gy holds g_alpha on entry
template <int HV>
__global__ void __launch_bounds__(256)
edge_gy_kernel(long count, int h, const int32_t *__restrict__ erow, const int32_t *__restrict__ col,
               const float *__restrict__ alpha, const uint8_t *__restrict__ mask, const float *__restrict__ s,
               const float *__restrict__ d, const float *__restrict__ sums, float slope, float *__restrict__ gy) {
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    long e; int pg;
    split_index(t, count, h / HV, e, pg);
    const int p0 = pg * HV;
    const int r = erow[e];
    bool pos[HV];
    if (mask) {
        if constexpr (HV == 4) {
            const uchar4 m = *reinterpret_cast<const uchar4 *>(mask + (size_t)e * h + p0);
            pos[0] = m.x != 0; pos[1] = m.y != 0; pos[2] = m.z != 0; pos[3] = m.w != 0;
        } else pos[0] = mask[(size_t)e * h + p0] != 0;
    } else {
        float sv[HV], dv[HV];
        load_vec<HV>(s + (size_t)r * h + p0, sv);
        load_vec<HV>(d + (size_t)col[e] * h + p0, dv);
#pragma unroll
        for (int i = 0; i < HV; ++i) pos[i] = (sv[i] + dv[i]) > 0.f;
    }
    float al[HV], g[HV];
    load_vec<HV>(alpha + (size_t)e * h + p0, al);
    load_vec<HV>(gy + (size_t)e * h + p0, g);
#pragma unroll
    for (int i = 0; i < HV; ++i) {
        const float ti = sums[((size_t)r * h + p0 + i) * 3];
        g[i] = al[i] * (g[i] - ti) * (pos[i] ? 1.f : slope);
    }
    store_vec<HV>(gy + (size_t)e * h + p0, g);
}

// ds_i = sum_e g_y_e = (1 - beta) (P_i - t_i Q_i): the softmax gradient sums to zero over a row,
// so only the entries with a positive logit (factor 1 instead of beta) leave a remainder.
// A row without stored entries has no sums (the row walk never visits it): its ds is zero.
__global__ void __launch_bounds__(256)
node_ds_kernel(long count, int h, const int32_t *__restrict__ rowptr, const float *__restrict__ sums, float slope,
               float *__restrict__ ds) {
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    const long i = t / h;
    if (rowptr[i] == rowptr[i + 1]) { ds[t] = 0.f; return; }
    const float ti = sums[t * 3], P = sums[t * 3 + 1], Q = sums[t * 3 + 2];
    ds[t] = (1.f - slope) * (P - ti * Q);
}

// dM_{i,p,c} += ds_{i,p} a_src_{p,c} + dd_{i,p} a_dst_{p,c}; one thread per VEC consecutive c
template <int VEC>
__global__ void __launch_bounds__(256)
add_rank1_kernel(long count, int h, int k, const float *__restrict__ ds, const float *__restrict__ dd,
                 const float *__restrict__ a_src, const float *__restrict__ a_dst, float *__restrict__ dM) {
    const long tv = (long)blockIdx.x * 256 + threadIdx.x;     // element t = VEC * tv = (i * h + p) * k + c
    if (tv >= count) return;
    const int kv = k / VEC, fv = h * kv;
    long ip, node;                                            // ip = i * h + p;  pcv = (p * k + c) / VEC
    int cv, pcv;
    split_index(tv, count, kv, ip, cv);
    split_index(tv, count, fv, node, pcv);
    const float a = ds[ip], b = dd[ip];
    float u[VEC], w[VEC], m[VEC];
    load_vec<VEC>(a_src + (size_t)pcv * VEC, u);
    load_vec<VEC>(a_dst + (size_t)pcv * VEC, w);
    load_vec<VEC>(dM + (size_t)tv * VEC, m);
#pragma unroll
    for (int i = 0; i < VEC; ++i) m[i] += a * u[i] + b * w[i];
    store_vec<VEC>(dM + (size_t)tv * VEC, m);
}

int pow2_at_least(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

template <class Op>
gnn_status_t run_head_walker(int nnz, int h, const int32_t *rowptr, const int32_t *erow, const int32_t *col, Op op,
                             float *out, float *part, hipStream_t st) {
    const int hp = pow2_at_least(h);
    const int seg = gat_segment_len(nnz, h);
    const long nseg = ceil_div(nnz, seg);
    const int gpb = 256 / hp;
    const int span = gpb * seg;
    const long nspan = ceil_div(nnz, span);
    const size_t lds = (size_t)2 * span * sizeof(int32_t) + (size_t)2 * 256 * Op::NACC * sizeof(float) +
                       (size_t)gpb * sizeof(WalkInfo);
    dim3 grid((unsigned)ceil_div(nseg, gpb)), fgrid((unsigned)ceil_div(nspan, 4));
#define WALK_CASE(HP_)                                                                                            \
    if (hp == HP_) {                                                                                              \
        hipLaunchKernelGGL((head_walker_kernel<Op, HP_, 8>), grid, dim3(256), lds, st, nnz, h, seg, nseg, erow,   \
                           col, op, out, part);                                                                   \
        GNN_TRY(launch_status());                                                                                 \
        hipLaunchKernelGGL((head_fixup_kernel<Op, HP_>), fgrid, dim3(256), 0, st, nnz, h, span, nspan, erow,      \
                           rowptr, part, out);                                                                    \
    }
    WALK_CASE(1) WALK_CASE(2) WALK_CASE(4) WALK_CASE(8) WALK_CASE(16) WALK_CASE(32) WALK_CASE(64)
#undef WALK_CASE
    return launch_status();
}

}  // namespace

// segment length of the head walker: GPB * seg <= 2048 staged entries, at least 16
int gat_segment_len(int64_t nnz, int h) {
    const int hp = pow2_at_least(h);
    const int64_t want_groups = 8192 * (kWave / hp);
    const int64_t seg = nnz / (want_groups > 0 ? want_groups : 1);
    const int cap = 8 * hp < 256 ? 8 * hp : 256;
    int p = 16;
    while (p * 2 <= seg && p * 2 <= cap) p <<= 1;
    return p;
}

size_t gat_walker_workspace_bytes(int64_t nnz, int h) {
    if (nnz <= 0) return kAlign;
    const int64_t span = (int64_t)(256 / pow2_at_least(h)) * gat_segment_len(nnz, h);
    return align_up((size_t)(2 * ceil_div(nnz, span)) * h * 3 * sizeof(float));
}

gnn_status_t gat_node_attention_launch(int n, int h, int k, const float *M, const float *a_src, const float *a_dst,
                                       float *s, float *d, hipStream_t st) {
    const long count = (long)n * h;
    if (count <= 0) return GNN_OK;
    if (k % 4 == 0 && aligned16(M) && aligned16(a_src) && aligned16(a_dst)) {
        int L = 1;                                          // lanes per (node, head): a power of two <= min(k / 4, 16)
        while (L < 16 && 8 * L <= k) L <<= 1;
#define NODE_ATT_CASE(L_)                                                                                         \
        if (L == L_)                                                                                              \
            hipLaunchKernelGGL((node_attention_kernel<4, L_>), dim3((unsigned)ceil_div(count * L_, 256)), dim3(256), \
                               0, st, count, h, k, M, a_src, a_dst, s, d);
        NODE_ATT_CASE(1) NODE_ATT_CASE(2) NODE_ATT_CASE(4) NODE_ATT_CASE(8) NODE_ATT_CASE(16)
#undef NODE_ATT_CASE
    } else {
        hipLaunchKernelGGL((node_attention_kernel<1, 1>), dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count,
                           h, k, M, a_src, a_dst, s, d);
    }
    return launch_status();
}

// stat [n][h][2] = (row max of the LeakyReLU'd logits, sum of exp(. - max))
gnn_status_t gat_edge_stats_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                   const int32_t *col, const float *s, const float *d, float slope, float *stat,
                                   void *workspace, hipStream_t st) {
    (void)n;
    if (nnz <= 0) return GNN_OK;
    StatsOp op{s, d, slope};
    return run_head_walker<StatsOp>(nnz, h, rowptr, erow, col, op, stat, static_cast<float *>(workspace), st);
}

// alpha_e = exp(w_e - max_i) / sum_i from the row statistics; mask_e = (y_e > 0) when asked for
gnn_status_t gat_edge_alpha_launch(int nnz, int h, const int32_t *erow, const int32_t *col, const float *s,
                                   const float *d, const float *stat, float slope, float *alpha, uint8_t *mask,
                                   hipStream_t st) {
    if (nnz <= 0) return GNN_OK;
    if (h % 4 == 0 && aligned16(s) && aligned16(d) && aligned16(stat) && aligned16(alpha) &&
        (!mask || (reinterpret_cast<uintptr_t>(mask) & 3u) == 0)) {
        const long count = (long)nnz * (h / 4);
        hipLaunchKernelGGL(edge_alpha_kernel<4>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count, h, erow,
                           col, s, d, stat, slope, alpha, mask);
    } else {
        const long count = (long)nnz * h;
        hipLaunchKernelGGL(edge_alpha_kernel<1>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count, h, erow,
                           col, s, d, stat, slope, alpha, mask);
    }
    return launch_status();
}

gnn_status_t gat_edge_softmax_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                     const int32_t *col, const float *s, const float *d, float slope, float *stat,
                                     float *alpha, uint8_t *mask, void *workspace, hipStream_t st) {
    GNN_TRY(gat_edge_stats_launch(n, nnz, h, rowptr, erow, col, s, d, slope, stat, workspace, st));
    return gat_edge_alpha_launch(nnz, h, erow, col, s, d, stat, slope, alpha, mask, st);
}

gnn_status_t sddmm_launch(int n, int nnz, const int32_t *erow, const int32_t *col, const float *val,
                          const float *B, const float *Ct, int heads, int f, float *D, hipStream_t st) {
    (void)n;
    const long count = (long)nnz * heads;
    if (count <= 0) return GNN_OK;
    const int vec = f % 4 == 0 && aligned16(B) && aligned16(Ct);
    if (vec && f >= 32) {
        // lanes per pair: a quarter of the feature count, 8 .. 32
        const int L = f >= 128 ? 32 : (f >= 64 ? 16 : 8);
        const dim3 grid((unsigned)ceil_div(count * L, 256));
        if (L == 32) hipLaunchKernelGGL(sddmm_coop_kernel<32>, grid, dim3(256), 0, st, count, heads, f, erow, col, val, B, Ct, D);
        else if (L == 16) hipLaunchKernelGGL(sddmm_coop_kernel<16>, grid, dim3(256), 0, st, count, heads, f, erow, col, val, B, Ct, D);
        else hipLaunchKernelGGL(sddmm_coop_kernel<8>, grid, dim3(256), 0, st, count, heads, f, erow, col, val, B, Ct, D);
        return launch_status();
    }
    hipLaunchKernelGGL(sddmm_edge_kernel, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count, heads, f,
                       erow, col, val, B, Ct, D, vec);
    return launch_status();
}

// gy [nnz][h]: g_alpha on entry, g_y on exit; sums [n][h][3] scratch; ds [n][h]
gnn_status_t gat_edge_backward_launch(int n, int nnz, int h, const int32_t *rowptr, const int32_t *erow,
                                      const int32_t *col, const float *alpha, const uint8_t *mask, const float *s,
                                      const float *d, float slope, float *gy, float *sums, float *ds,
                                      void *workspace, hipStream_t st) {
    if (n <= 0) return GNN_OK;
    if (nnz <= 0) return fill_zero_launch((int64_t)n * h, ds, st);     // no entries: every row sum is empty
    SumsOp op{alpha, gy, mask, s, d};
    GNN_TRY(run_head_walker<SumsOp>(nnz, h, rowptr, erow, col, op, sums, static_cast<float *>(workspace), st));
    const long ecount = (long)nnz * h, ncount = (long)n * h;
    if (h % 4 == 0 && aligned16(alpha) && aligned16(gy) && aligned16(s) && aligned16(d) &&
        (!mask || (reinterpret_cast<uintptr_t>(mask) & 3u) == 0))
        hipLaunchKernelGGL(edge_gy_kernel<4>, dim3((unsigned)ceil_div(ecount / 4, 256)), dim3(256), 0, st, ecount / 4, h,
                           erow, col, alpha, mask, s, d, sums, slope, gy);
    else
        hipLaunchKernelGGL(edge_gy_kernel<1>, dim3((unsigned)ceil_div(ecount, 256)), dim3(256), 0, st, ecount, h, erow,
                           col, alpha, mask, s, d, sums, slope, gy);
    GNN_TRY(launch_status());
    hipLaunchKernelGGL(node_ds_kernel, dim3((unsigned)ceil_div(ncount, 256)), dim3(256), 0, st, ncount, h, rowptr, sums,
                       slope, ds);
    return launch_status();
}

gnn_status_t gat_add_rank1_launch(int n, int h, int k, const float *ds, const float *dd, const float *a_src,
                                  const float *a_dst, float *dM, hipStream_t st) {
    const long count = (long)n * h * k;
    if (count <= 0) return GNN_OK;
    if (k % 4 == 0 && aligned16(dM) && aligned16(a_src) && aligned16(a_dst))
        hipLaunchKernelGGL(add_rank1_kernel<4>, dim3((unsigned)ceil_div(count / 4, 256)), dim3(256), 0, st, count / 4, h,
                           k, ds, dd, a_src, a_dst, dM);
    else
        hipLaunchKernelGGL(add_rank1_kernel<1>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, st, count, h, k, ds,
                           dd, a_src, a_dst, dM);
    return launch_status();
}

}  // namespace gnn
