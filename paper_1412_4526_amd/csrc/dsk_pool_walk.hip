// Stride-1 pooling with d-regularly sparse 2 x 2 and 3 x 3 kernels (paper Sec. 3.1-3.2;
// backward Sec. 4.2): the kernels the benchmark networks spend their pooling time in.
//
// A thread owns V = 4 neighbouring columns (16 bytes in fp32, 8 in bf16) and WALKS
// DOWN one residue class of rows modulo d (rows u, u+d, u+2d, ...): the k tap rows of
// an output row are the next rows of the same class, so what the thread computed from
// the previous k-1 input rows stays in registers and every input row is loaded once
// per walk, not once per tile of 8 rows.  A class is cut into segments of at most 64
// rows (one thread each), which costs (k-1)/64 re-reads.  Every memory instruction
// moves four pixels per lane (tap indices: 4 bytes): the vector memory path takes as
// long for a 4-byte access per lane as for a 16-byte one.
//
// Max-pool ties: taps are ranked by a*k+b and only a strictly greater value replaces
// the running maximum, so the lowest index wins: first maximum of each input row, then
// the first row holding the overall maximum.
//
// The backward kernels are the gather form (each dx element inspects its k*k candidate
// outputs: no atomics, fixed summation order).  FUSE: the error map that leaves the
// pool is the one that enters the non-linearity of the convolution before it, so
// act'(y) is applied before the store and the bias gradient of that convolution (the
// sum of the stored map, Sec. 4.1) is collected in the same pass.
#include <type_traits>

#include "dsk_internal.h"

namespace dsk {

static constexpr int kWT = 256;
static constexpr int kSegRows = 64;
static constexpr long kFillThreads = 2048L * 256;      // threads wanted in flight: eight workgroups per CU
// cache policy (the aux operand of the buffer builtins) of the loads and of the stores.  Non-temporal accesses (2)
// were measured: loads lose 10-20 % (neighbouring lanes and tap columns share lines), stores gain 1 % on maps whose
// rows are 16-byte aligned and lose 5-15 % on the others.
static constexpr int kAuxLd = 0, kAuxSt = 0;

typedef float wf4 __attribute__((ext_vector_type(4)));
typedef unsigned wu4 __attribute__((ext_vector_type(4)));
typedef unsigned wu2 __attribute__((ext_vector_type(2)));

struct WalkShape {
    int planes, H, W, Ho, Wo, d;
    int J, nseg;               // rows of a class one thread walks over; segments per class
    int lanes;                 // threads side by side along a row: ceil(columns / V)
    int row_groups;            // (segment, class) pairs: walks per column group
    int bpp;                   // workgroups per plane
    long n_blocks;
};

// Thread t of a plane takes walk t / lanes, column group t % lanes: consecutive threads lie side by side along
// a row (a workgroup reads and writes runs of 4 KB), consecutive walks are the d classes of one segment
// (neighbouring rows), and no lane is idle but in the last workgroup of a plane.
template <int V>
__device__ inline bool walk_decode(const WalkShape &s, int &plane, int &res, int &j0, int &col)
{
    plane = (int)(blockIdx.x / (unsigned)s.bpp);
    const int t = (int)(blockIdx.x % (unsigned)s.bpp) * kWT + (int)threadIdx.x;
    const int rg = t / s.lanes;
    res = rg % s.d;
    j0 = (rg / s.d) * s.J;
    col = (t - rg * s.lanes) * V;
    return rg < s.row_groups;
}

// V consecutive elements from element offset `off` of the plane (16 bytes; any alignment)
template <int V>
__device__ inline void wld(BufRsrc r, const float *, unsigned off, float (&o)[V])
{
    static_assert(V == 4, "four fp32 pixels per access");
    const wf4 t = __builtin_bit_cast(wf4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(off * 4u), 0, kAuxLd));
    o[0] = t[0]; o[1] = t[1]; o[2] = t[2]; o[3] = t[3];
}
template <int V>
__device__ inline void wld(BufRsrc r, const bf16 *, unsigned off, float (&o)[V])
{
    static_assert(V == 4 || V == 8, "four or eight bf16 pixels per access");
    unsigned t[V / 2];
    if constexpr (V == 4) {
        const wu2 q = __builtin_amdgcn_raw_buffer_load_b64(r, (int)(off * 2u), 0, kAuxLd);
        t[0] = q[0]; t[1] = q[1];
    } else {
        const wu4 q = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(off * 2u), 0, kAuxLd);
        t[0] = q[0]; t[1] = q[1]; t[2] = q[2]; t[3] = q[3];
    }
#pragma unroll
    for (int i = 0; i < V / 2; ++i) {
        o[2 * i] = __builtin_bit_cast(float, t[i] << 16);
        o[2 * i + 1] = __builtin_bit_cast(float, t[i] & 0xffff0000u);
    }
}
// stores V elements; v returns what was stored (bf16: the rounded values)
template <int V>
__device__ inline void wst(BufRsrc r, float *, unsigned off, float (&v)[V])
{
    const wf4 t = {v[0], v[1], v[2], v[3]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(wu4, t), r, (int)(off * 4u), 0, kAuxSt);
}
template <int V>
__device__ inline void wst(BufRsrc r, bf16 *, unsigned off, float (&v)[V])
{
    unsigned h[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        h[j] = f32_to_bf16(v[j]).v;
        v[j] = __builtin_bit_cast(float, h[j] << 16);
    }
    if constexpr (V == 4) {
        const wu2 t = {h[0] | h[1] << 16, h[2] | h[3] << 16};
        __builtin_amdgcn_raw_buffer_store_b64(t, r, (int)(off * 2u), 0, kAuxSt);
    } else {
        const wu4 t = {h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16};
        __builtin_amdgcn_raw_buffer_store_b128(t, r, (int)(off * 2u), 0, kAuxSt);
    }
}
__device__ inline float round_as(const float *, float v) { return v; }
__device__ inline float round_as(const bf16 *, float v) { return bf16_to_f32(f32_to_bf16(v)); }

// V tap indices, one per byte: packed in V/4 words
template <int V> struct TapWords { unsigned w[V / 4]; };
template <int V>
__device__ inline TapWords<V> wld_idx(BufRsrc r, unsigned off)
{
    TapWords<V> t;
    if constexpr (V == 4) {
        t.w[0] = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, kAuxLd);
    } else {
        const wu2 q = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, kAuxLd);
        t.w[0] = q[0]; t.w[1] = q[1];
    }
    return t;
}
template <int V>
__device__ inline void wst_idx(BufRsrc r, unsigned off, const int (&bi)[V])
{
    unsigned w[V / 4];
#pragma unroll
    for (int i = 0; i < V / 4; ++i)
        w[i] = (unsigned)bi[4 * i] | (unsigned)bi[4 * i + 1] << 8 | (unsigned)bi[4 * i + 2] << 16 | (unsigned)bi[4 * i + 3] << 24;
    if constexpr (V == 4) {
        __builtin_amdgcn_raw_buffer_store_b32(w[0], r, (int)off, 0, kAuxSt);
    } else {
        const wu2 q = {w[0], w[1]};
        __builtin_amdgcn_raw_buffer_store_b64(q, r, (int)off, 0, kAuxSt);
    }
}
template <int V>
__device__ inline int tap_of(const TapWords<V> &t, int j) { return (int)((t.w[j / 4] >> (8 * (j % 4))) & 0xffu); }

// The same V elements one by one, for the rows at the two ends of a plane: a 16-byte access there may begin
// before the plane or reach past its end, and the range check of the buffer returns zero for every 32-bit
// word that is not wholly inside -- also for its part that is (a bf16 pixel or a tap index next to the end).
// Elements outside [0, n) read as zero.
template <typename T, int V>
__device__ inline void wld_edge(BufRsrc r, const T *p, int off, int n, float (&o)[V])
{
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const bool ok = off + j >= 0 && off + j < n;
        const float v = buf_ld(r, p, ok ? (unsigned)(off + j) : 0u, 0u);
        o[j] = ok ? v : 0.f;
    }
}
template <int V>
__device__ inline TapWords<V> wld_idx_edge(BufRsrc r, const uint8_t *p, int off, int n)
{
    TapWords<V> t;
#pragma unroll
    for (int i = 0; i < V / 4; ++i) t.w[i] = 0u;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const bool ok = off + j >= 0 && off + j < n;
        const unsigned v = (unsigned)buf_ld(r, p, ok ? (unsigned)(off + j) : 0u, 0u);
        t.w[j / 4] |= (ok ? v : 0xffu) << (8 * (j % 4));
    }
    return t;
}

// one input row: first maximum (or sum) over the K tap columns, per owned column
template <int K, bool IS_MAX, int V>
__device__ inline void walk_row(const float (&xv)[K][V], float (&rv)[V], int (&rb)[V])
{
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float best = xv[0][j];
        int bi = 0;
#pragma unroll
        for (int b = 1; b < K; ++b) {
            if (IS_MAX) {
                if (xv[b][j] > best) { best = xv[b][j]; bi = b; }
            } else {
                best += xv[b][j];
            }
        }
        rv[j] = best;
        rb[j] = bi;
    }
}

// Descriptors reach from (a little before) the plane to the END OF THE TENSOR, so that a 16-byte access of an
// ordinary row may begin in the previous row or end in the next one (also across planes: what it brings from
// there is masked or never stored).  Only a batch of rows that touches the first rows of the first plane or the
// last row of the last plane is read pixel by pixel (EDGE; see wld_edge): a different body of the loop, chosen
// per batch, so that the ordinary body has no branch between its loads.
//
// R: output rows per batch of loads
template <typename T, int K, bool IS_MAX, int V, int R>
__global__ void __launch_bounds__(kWT)
pool_walk_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, WalkShape s)
{
    int plane, res, j0, v;
    if (!walk_decode<V>(s, plane, res, j0, v)) return;
    const int njo = res < s.Ho ? (s.Ho - res + s.d - 1) / s.d : 0;      // output rows of this class
    if (j0 >= njo || v >= s.Wo) return;
    const int jend = j0 + s.J < njo ? j0 + s.J : njo;
    const bool last_plane = plane == s.planes - 1;
    const T *xp = x + (long)plane * s.H * s.W;
    const BufRsrc rx = buf_rsrc(xp, x + (long)s.planes * s.H * s.W);
    T *yp = y + (long)plane * s.Ho * s.Wo;
    const BufRsrc ry = buf_rsrc(yp, yp + (long)s.Ho * s.Wo);
    uint8_t *ap = IS_MAX && am ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc ra = buf_rsrc(ap, ap + (ap ? (long)s.Ho * s.Wo : 0));
    const bool whole = v + V <= s.Wo;      // columns beyond the map are computed from whatever the loads bring, never stored
    // what the previous K-1 input rows gave: value and tap column per owned output column
    float cv[K - 1][V];
    int cb[K - 1][V];
    {
        // (these rows are never the plane's last one: the output row j0 has K-1 more tap rows below them)
        float xv[K - 1][K][V];
#pragma unroll
        for (int t = 0; t < K - 1; ++t)
#pragma unroll
            for (int b = 0; b < K; ++b) wld<V>(rx, xp, (unsigned)((res + (j0 + t) * s.d) * s.W + v + b * s.d), xv[t][b]);
#pragma unroll
        for (int t = 0; t < K - 1; ++t) walk_row<K, IS_MAX, V>(xv[t], cv[t], cb[t]);
    }
    auto batch = [&](int jc, auto edge) __attribute__((always_inline)) {
        constexpr bool EDGE = decltype(edge)::value;
        float xv[R][K][V];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            int row = res + (jc + i + K - 1) * s.d;
            row = row < s.H ? row : s.H - 1;      // past the last output row: loaded, never used
#pragma unroll
            for (int b = 0; b < K; ++b) {
                if constexpr (EDGE) wld_edge<T, V>(rx, xp, row * s.W + v + b * s.d, s.H * s.W, xv[i][b]);
                else wld<V>(rx, xp, (unsigned)(row * s.W + v + b * s.d), xv[i][b]);
            }
        }
        // the values are pinned here so that the loads of a batch are issued together above, not one by one
        // where the comparisons below use them
#pragma unroll
        for (int i = 0; i < R; ++i)
#pragma unroll
            for (int b = 0; b < K; ++b)
#pragma unroll
                for (int j = 0; j < V; ++j) asm volatile("" : "+v"(xv[i][b][j]));
#pragma unroll
        for (int i = 0; i < R; ++i) {
            float nv[V];
            int nb[V];
            walk_row<K, IS_MAX, V>(xv[i], nv, nb);
            const int jo = jc + i;
            if (jo < jend) {
                float best[V];
                int bi[V];
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    best[j] = cv[0][j];
                    bi[j] = cb[0][j];
#pragma unroll
                    for (int a = 1; a < K; ++a) {
                        const float val = a < K - 1 ? cv[a < K - 1 ? a : 0][j] : nv[j];
                        const int idx = a < K - 1 ? cb[a < K - 1 ? a : 0][j] : nb[j];
                        if (IS_MAX) {
                            if (val > best[j]) { best[j] = val; bi[j] = a * K + idx; }
                        } else {
                            best[j] += val;
                        }
                    }
                    if (!IS_MAX) best[j] *= 1.0f / (float)(K * K);
                }
                const unsigned o = (unsigned)((res + jo * s.d) * s.Wo) + (unsigned)v;
                if (whole) {
                    wst<V>(ry, yp, o, best);
                    if (ap) wst_idx<V>(ra, o, bi);
                } else {
#pragma unroll
                    for (int j = 0; j < V; ++j)
                        if (v + j < s.Wo) {
                            buf_st(ry, yp, o + j, 0u, best[j]);
                            if (ap) buf_st(ra, ap, o + j, 0u, bi[j]);
                        }
                }
            }
#pragma unroll
            for (int a = 0; a + 1 < K - 1; ++a)
#pragma unroll
                for (int j = 0; j < V; ++j) { cv[a][j] = cv[a + 1][j]; cb[a][j] = cb[a + 1][j]; }
#pragma unroll
            for (int j = 0; j < V; ++j) { cv[K - 2][j] = nv[j]; cb[K - 2][j] = nb[j]; }
        }
    };
    for (int jc = j0; jc < jend; jc += R) {
        // an access of the batch could end past the last plane (decided for the whole wave: the lanes of a wave may
        // be on different walks)
        const int row_max = res + (jc + R - 1 + K - 1) * s.d < s.H ? res + (jc + R - 1 + K - 1) * s.d : s.H - 1;
        if (__any(last_plane && (long)row_max * s.W + s.W + V > (long)s.H * s.W)) batch(jc, std::true_type{});
        else batch(jc, std::false_type{});
    }
}

// One dy row as the dx columns q .. q+V-1 see it: for tap column b the dy columns q - b*d .. + V-1 (zero where
// they do not exist) and their tap indices.
template <int K, int V>
struct GradRow {
    float g[K][V];
    TapWords<V> t[K];
};

// dx rows of one class (class-local index jp, row res + jp*d) collect from dy rows jp - a of the same class.
template <typename T, int K, bool IS_MAX, int V, int R, bool FUSE>
__global__ void __launch_bounds__(kWT)
pool_walk_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx,
                     const T *__restrict__ yprev, float *__restrict__ part, int act, WalkShape s)
{
    __shared__ float red[kWT / 64];
    int plane, res, j0, q;
    const bool decoded = walk_decode<V>(s, plane, res, j0, q);
    const int njp = res < s.H ? (s.H - res + s.d - 1) / s.d : 0;        // dx rows of this class
    const int nju = res < s.Ho ? (s.Ho - res + s.d - 1) / s.d : 0;      // dy rows of this class
    const bool active = decoded && j0 < njp && q < s.W;
    float bias_acc = 0.f;
    if (active) {
        const int jend = j0 + s.J < njp ? j0 + s.J : njp;
        const bool last_plane = plane == s.planes - 1;
        // the descriptors of dy and of the tap indices begin `lead` entries before the plane (but never before the
        // tensor), so that the accesses of the tap columns to the left of the first columns stay non-negative
        const long hw_o = (long)s.Ho * s.Wo, hw = (long)s.H * s.W;
        const int lead = (long)plane * hw_o < (long)(K - 1) * s.d ? (int)(plane * hw_o) : (K - 1) * s.d;      // never before the tensor
        const T *dyp = dy + (long)plane * hw_o - lead;
        const uint8_t *amp = IS_MAX ? am + (long)plane * hw_o - lead : nullptr;
        const BufRsrc rg = buf_rsrc(dyp, dy + (long)s.planes * hw_o);
        const BufRsrc ra = buf_rsrc(amp, IS_MAX ? am + (long)s.planes * hw_o : amp);
        T *dxp = dx + (long)plane * hw;
        const BufRsrc rd = buf_rsrc(dxp, dxp + hw);
        const T *ypp = FUSE && act != DSK_ACT_NONE ? yprev + (long)plane * hw : nullptr;
        const BufRsrc ry = buf_rsrc(ypp, ypp ? yprev + (long)s.planes * hw : ypp);
        const bool whole = q + V <= s.W;
        // per tap column b: first dy column, and which of its V columns exist
        int c0[K];
        unsigned cok[K];
#pragma unroll
        for (int b = 0; b < K; ++b) {
            c0[b] = q - b * s.d;
            cok[b] = 0;
#pragma unroll
            for (int j = 0; j < V; ++j) cok[b] |= (c0[b] + j >= 0 && c0[b] + j < s.Wo) ? 1u << j : 0u;
        }
        // one dy row (rows that do not exist are read from row 0 and masked); returns whether the row exists
        auto load_row = [&](int ju, GradRow<K, V> &r, auto edge) __attribute__((always_inline)) {
            constexpr bool EDGE = decltype(edge)::value;
            const bool row_ok = ju >= 0 && ju < nju;
            const int ro = (row_ok ? res + ju * s.d : 0) * s.Wo;
#pragma unroll
            for (int b = 0; b < K; ++b) {
                if constexpr (EDGE) {
                    wld_edge<T, V>(rg, dyp, lead + ro + c0[b], lead + (int)hw_o, r.g[b]);
                    if (IS_MAX) r.t[b] = wld_idx_edge<V>(ra, amp, lead + ro + c0[b], lead + (int)hw_o);
                } else {
                    wld<V>(rg, dyp, (unsigned)(lead + ro + c0[b]), r.g[b]);
                    if (IS_MAX) r.t[b] = wld_idx<V>(ra, (unsigned)(lead + ro + c0[b]));
                }
            }
            return row_ok;
        };
        auto mask_row = [&](GradRow<K, V> &r, bool row_ok) __attribute__((always_inline)) {
#pragma unroll
            for (int b = 0; b < K; ++b)
#pragma unroll
                for (int j = 0; j < V; ++j) r.g[b][j] = row_ok && ((cok[b] >> j) & 1u) ? r.g[b][j] : 0.f;
        };
        // a batch of dy rows ju0 .. ju0+n-1 needs the pixel-by-pixel form if one of its accesses could begin
        // before the first plane or end past the last one
        auto is_edge = [&](int ju0, int n) {
            bool e = false;
            for (int t = 0; t < n; ++t) {
                const int ju = ju0 + t;
                const int ro = (ju >= 0 && ju < nju ? res + ju * s.d : 0) * s.Wo;
                e |= lead + ro < (K - 1) * s.d || (last_plane && (long)ro + s.W + V > hw_o);
            }
            return e;
        };
        GradRow<K, V> carry[K - 1];      // dy rows jp-(K-1) .. jp-1, oldest first
        if (__any(is_edge(j0 - (K - 1), K - 1))) {
#pragma unroll
            for (int t = 0; t < K - 1; ++t) mask_row(carry[t], load_row(j0 - (K - 1) + t, carry[t], std::true_type{}));
        } else {
#pragma unroll
            for (int t = 0; t < K - 1; ++t) mask_row(carry[t], load_row(j0 - (K - 1) + t, carry[t], std::false_type{}));
        }
        auto batch = [&](int jc, auto edge) __attribute__((always_inline)) {
            constexpr bool EDGE = decltype(edge)::value;
            GradRow<K, V> nr[R];
            bool nok[R];
            float yv[R][V];
#pragma unroll
            for (int i = 0; i < R; ++i) {
                nok[i] = load_row(jc + i, nr[i], edge);
                if (FUSE && ypp) {
                    int p = res + (jc + i) * s.d;
                    p = p < s.H ? p : s.H - 1;
                    if constexpr (EDGE) wld_edge<T, V>(ry, ypp, p * s.W + q, (int)hw, yv[i]);
                    else wld<V>(ry, ypp, (unsigned)(p * s.W + q), yv[i]);
                }
            }
            // pinned: the loads of a batch are issued together above
#pragma unroll
            for (int i = 0; i < R; ++i) {
#pragma unroll
                for (int b = 0; b < K; ++b) {
#pragma unroll
                    for (int j = 0; j < V; ++j) asm volatile("" : "+v"(nr[i].g[b][j]));
                    if (IS_MAX) {
#pragma unroll
                        for (int w = 0; w < V / 4; ++w) asm volatile("" : "+v"(nr[i].t[b].w[w]));
                    }
                }
                if (FUSE && ypp) {
#pragma unroll
                    for (int j = 0; j < V; ++j) asm volatile("" : "+v"(yv[i][j]));
                }
            }
#pragma unroll
            for (int i = 0; i < R; ++i) {
                mask_row(nr[i], nok[i]);
                const int jp = jc + i;
                if (jp < jend) {
                    float acc[V];
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        acc[j] = 0.f;
#pragma unroll
                        for (int a = K - 1; a >= 0; --a) {      // dy row jp - a: the carried rows, then the new one
                            const GradRow<K, V> &r = a > 0 ? carry[a > 0 ? K - 1 - a : 0] : nr[i];
#pragma unroll
                            for (int b = 0; b < K; ++b)
                                acc[j] += !IS_MAX || tap_of<V>(r.t[b], j) == a * K + b ? r.g[b][j] : 0.f;
                        }
                        if (!IS_MAX) acc[j] *= 1.0f / (float)(K * K);
                        if (FUSE && ypp)
                            acc[j] *= act == DSK_ACT_RELU ? (yv[i][j] > 0.f ? 1.f : 0.f) : 1.f - yv[i][j] * yv[i][j];
                    }
                    const unsigned o = (unsigned)((res + jp * s.d) * s.W + q);
                    if (whole) {
                        wst<V>(rd, dxp, o, acc);
#pragma unroll
                        for (int j = 0; j < V; ++j) bias_acc += acc[j];
                    } else {
#pragma unroll
                        for (int j = 0; j < V; ++j)
                            if (q + j < s.W) {
                                buf_st(rd, dxp, o + j, 0u, acc[j]);
                                bias_acc += round_as(dxp, acc[j]);
                            }
                    }
                }
#pragma unroll
                for (int a = 0; a + 1 < K - 1; ++a) carry[a] = carry[a + 1];
                carry[K - 2] = nr[i];
            }
        };
        for (int jc = j0; jc < jend; jc += R) {
            // (y: the batch that reaches the last dx rows of the last plane)
            const int p_max = res + (jc + R - 1) * s.d < s.H ? res + (jc + R - 1) * s.d : s.H - 1;
            if (__any(is_edge(jc, R) || (FUSE && last_plane && (long)p_max * s.W + s.W + V > hw))) batch(jc, std::true_type{});
            else batch(jc, std::false_type{});
        }
    }
    if (FUSE) {
        // the workgroup's share of the bias gradient: wavefront shuffles, then LDS, in a fixed order
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) bias_acc += __shfl_down(bias_acc, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = bias_acc;
        __syncthreads();
        if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
    }
}

// db[f] = sum over images and workgroups of a plane, in index order
__global__ void __launch_bounds__(kWT)
pool_bias_sum_kernel(const float *__restrict__ part, float *__restrict__ db, int N, int C, int bpp)
{
    __shared__ float red[kWT];
    const int f = blockIdx.x;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) {
        const float *src = part + ((long)n * C + f) * bpp;
        for (int t = threadIdx.x; t < bpp; t += kWT) acc += src[t];
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kWT / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) db[f] = red[0];
}

// rows / cols: extent of the map the threads are spread over (the output of the kernel)
static WalkShape make_walk(int N, int C, int H, int W, int k, int d, int rows, int cols, int V, int R)
{
    WalkShape s{};
    s.planes = N * C;
    s.H = H; s.W = W;
    s.Ho = H - (k - 1) * d; s.Wo = W - (k - 1) * d;
    s.d = d;
    const int nj = (rows + d - 1) / d;      // rows of the longest class
    s.lanes = (cols + V - 1) / V;
    // segments of at most kSegRows rows -- shorter ones (down to one batch of R rows) on small maps, so that there
    // are enough threads to fill the chip: a walk re-reads k-1 rows per segment
    s.nseg = (nj + kSegRows - 1) / kSegRows;
    const long want = (kFillThreads + (long)s.planes * d * s.lanes - 1) / ((long)s.planes * d * s.lanes);
    if (s.nseg < want) s.nseg = (int)(want < (nj + R - 1) / R ? want : (nj + R - 1) / R);
    if (s.nseg < 1) s.nseg = 1;
    s.J = ((nj + s.nseg - 1) / s.nseg + R - 1) / R * R;
    s.nseg = (nj + s.J - 1) / s.J;
    s.row_groups = d * s.nseg;
    s.bpp = (int)(((long)s.row_groups * s.lanes + kWT - 1) / kWT);
    s.n_blocks = (long)s.planes * s.bpp;
    return s;
}

// rows per batch of loads: what the registers hold
static constexpr int walk_rows(int k, bool) { return k == 2 ? 8 : 4; }
// the gradient kernels hold two or three times as much per row (values and tap indices of k tap columns, and y)
static constexpr int walk_rows_bwd(int k, int v) { return (k == 2 ? 16 : 8) / v; }
// pixels per access in the gradient kernels: 16 bytes in both types
static constexpr int walk_v_bwd(dsk_dtype t) { return t == DSK_F32 ? 4 : 8; }

bool pool_walk_ok(int N, int C, int H, int W, int k, int d, dsk_dtype t)
{
    if (k != 2 && k != 3) return false;
    const int V = walk_v_bwd(t), R = walk_rows_bwd(k, V);
    return make_walk(N, C, H, W, k, d, H, W, V, R).n_blocks < 0x7fffffffL;      // the gradient's grid is the larger one
}

template <typename T, bool IS_MAX, int V>
static int walk_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d, hipStream_t st)
{
    constexpr bool B16 = sizeof(T) == 2;
    const WalkShape s = make_walk(N, C, H, W, k, d, H - (k - 1) * d, W - (k - 1) * d, V, walk_rows(k, B16));
    const dim3 grid((unsigned)s.n_blocks), block(kWT);
    if (k == 2) pool_walk_fwd_kernel<T, 2, IS_MAX, V, walk_rows(2, B16)><<<grid, block, 0, st>>>((const T *)x, (T *)y, am, s);
    else pool_walk_fwd_kernel<T, 3, IS_MAX, V, walk_rows(3, B16)><<<grid, block, 0, st>>>((const T *)x, (T *)y, am, s);
    return check_launch();
}

int launch_pool_walk_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d, bool is_max,
                         dsk_dtype t, hipStream_t st)
{
    if (t == DSK_F32)
        return is_max ? walk_fwd<float, true, 4>(x, y, am, N, C, H, W, k, d, st)
                      : walk_fwd<float, false, 4>(x, y, am, N, C, H, W, k, d, st);
    return is_max ? walk_fwd<bf16, true, 4>(x, y, am, N, C, H, W, k, d, st)
                  : walk_fwd<bf16, false, 4>(x, y, am, N, C, H, W, k, d, st);
}

size_t pool_bwd_act_bias_ws_bytes(int N, int C, int H, int W, int k, int d, dsk_dtype t)
{
    const WalkShape s = make_walk(N, C, H, W, k, d, H, W, walk_v_bwd(t), walk_rows_bwd(k, walk_v_bwd(t)));
    return (size_t)s.n_blocks * sizeof(float);
}

template <typename T, bool IS_MAX, int V>
static int walk_bwd(const void *dy, const uint8_t *am, void *dx, const void *yprev, float *db, int act, void *ws,
                    int N, int C, int H, int W, int k, int d, hipStream_t st)
{
    const WalkShape s = make_walk(N, C, H, W, k, d, H, W, V, walk_rows_bwd(k, V));
    const dim3 grid((unsigned)s.n_blocks), block(kWT);
    float *part = (float *)ws;
    const bool fuse = db != nullptr;
#define DSK_WB(KK, FU) pool_walk_bwd_kernel<T, KK, IS_MAX, V, walk_rows_bwd(KK, V), FU><<<grid, block, 0, st>>>( \
        (const T *)dy, am, (T *)dx, (const T *)yprev, part, act, s)
    if (k == 2 && fuse) DSK_WB(2, true);
    else if (k == 2) DSK_WB(2, false);
    else if (fuse) DSK_WB(3, true);
    else DSK_WB(3, false);
#undef DSK_WB
    if (fuse) pool_bias_sum_kernel<<<dim3((unsigned)C), block, 0, st>>>(part, db, N, C, s.bpp);
    return check_launch();
}

// db == nullptr: the plain pool gradient.  Otherwise dx = pool gradient * act'(yprev) and db[c] = sum of dx over
// images and pixels (yprev is not read for DSK_ACT_NONE).
int launch_pool_walk_bwd(const void *dy, const uint8_t *am, void *dx, const void *yprev, float *db, int act, void *ws,
                         int N, int C, int H, int W, int k, int d, bool is_max, dsk_dtype t, hipStream_t st)
{
    if (t == DSK_F32)
        return is_max ? walk_bwd<float, true, 4>(dy, am, dx, yprev, db, act, ws, N, C, H, W, k, d, st)
                      : walk_bwd<float, false, 4>(dy, am, dx, yprev, db, act, ws, N, C, H, W, k, d, st);
    return is_max ? walk_bwd<bf16, true, 8>(dy, am, dx, yprev, db, act, ws, N, C, H, W, k, d, st)
                  : walk_bwd<bf16, false, 8>(dy, am, dx, yprev, db, act, ws, N, C, H, W, k, d, st);
}

} // namespace dsk
