// Video (3-D) layers: the method carried over to video with 3-D convolution and 3-D pooling, which the paper's
// closing section proposes (Sec. 6).  A strided 3-D layer of a cube classifier becomes a stride-1 layer whose
// kernel is sparse in time as well: taps dt frames apart and d pixels apart (Algorithm 1 applied to the
// temporal axis with the temporal strides, and to the spatial axes with the spatial ones).
//
// Maps are stored frame-major, [N][T][C][H][W]: every frame is an image [C][H][W], so a video is a batch of
// T images and all per-pixel work (non-linearity, loss, padding) is the 2-D call on N*T images.  A 3-D
// convolution is then a 2-D sparse convolution of every output frame whose contraction also runs over the kt
// temporal taps: the planes of tap e are the C planes of the frame e*dt further on.  The 2-D matrix-core
// kernels take such "grouped" planes (ConvShape), so a layer costs one launch (forward), kt launches (weight
// gradient: one 2-D weight gradient per temporal tap, each over all frames), or, per video, one launch for every
// run of frames that are reached by the same temporal taps (backward-data).
//
// Weights are [kt][K][C][kh][kw]: a temporal tap's 2-D kernel is contiguous, which is what the weight gradient
// writes and what backward-data reads (in reversed tap order); forward re-orders them once per call.
#include "dsk_internal.h"

namespace dsk {

namespace {

constexpr int kThreads = 256;

struct Conv3 {
    int N, T, C, H, W, K, kt, kh, kw, dt, d, To, Ho, Wo;
    long taps() const { return (long)kh * kw; }
    long frame_in() const { return (long)C * H * W; }
    long frame_out() const { return (long)K * Ho * Wo; }
    long w2d() const { return (long)K * C * kh * kw; }      // one temporal tap's kernel
};

inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// forward: wf[f][e*C + c][t] = w[e][f][c][t]
__global__ void __launch_bounds__(kThreads)
w3_forward_order_kernel(const float *__restrict__ w, float *__restrict__ wf, int kt, int K, int C, int taps)
{
    const long total = (long)kt * K * C * taps;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int t = (int)(idx % taps);
    const int c = (int)((idx / taps) % C);
    const int e = (int)((idx / ((long)taps * C)) % kt);
    const int f = (int)(idx / ((long)taps * C * kt));
    wf[idx] = w[(((long)e * K + f) * C + c) * taps + t];
}

// backward-data: wr[r][f][c][t] = w[kt-1-r][f][c][t]
__global__ void __launch_bounds__(kThreads)
w3_reverse_kernel(const float *__restrict__ w, float *__restrict__ wr, int kt, long per_tap)
{
    const long total = (long)kt * per_tap;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int r = (int)(idx / per_tap);
    wr[idx] = w[(long)(kt - 1 - r) * per_tap + (idx - (long)r * per_tap)];
}

template <typename T>
__global__ void __launch_bounds__(kThreads)
fill_zero_kernel(T *__restrict__ p, long count)
{
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx < count) stf(p, idx, 0.f);
}

// xp[n][t][c][p][q] = x[n][t-tlo][c][p-lo][q-lo], zero outside (the padding of Sec. 3.3 on all three axes)
template <typename TO>
__global__ void __launch_bounds__(kThreads)
pad_video_kernel(const float *__restrict__ x, TO *__restrict__ xp, int N, int T, int C, int H, int W, int tlo, int lo,
                 int Tp, int Hp, int Wp)
{
    const long total = (long)N * Tp * C * Hp * Wp;
    long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const long o = idx;
    const int q = (int)(idx % Wp) - lo; idx /= Wp;
    const int p = (int)(idx % Hp) - lo; idx /= Hp;
    const int c = (int)(idx % C); idx /= C;
    const int t = (int)(idx % Tp) - tlo;
    const int n = (int)(idx / Tp);
    float v = 0.f;
    if (t >= 0 && t < T && p >= 0 && p < H && q >= 0 && q < W) v = x[((((long)n * T + t) * C + c) * H + p) * W + q];
    stf(xp, o, v);
}

inline unsigned blocks_for(long total) { return (unsigned)((total + kThreads - 1) / kThreads); }

// the 2-D call that computes every output frame of the forward pass
ConvShape fwd_shape(const Conv3 &c)
{
    ConvShape s{c.N * c.To, c.kt * c.C, c.H, c.W, c.K, c.kh, c.kw, c.d, c.Ho, c.Wo};
    if (c.kt > 1) {
        s.gsize = c.C;
        s.gjump = (long)(c.dt - 1) * c.frame_in();
        s.bgroup = c.To;
        s.bskip = c.T - c.To;
        s.in_extent = (long)c.N * c.T * c.frame_in();
    }
    return s;
}

// the 2-D weight gradient of temporal tap e (x begins e*dt frames into the first video)
ConvShape bww_shape(const Conv3 &c, int e)
{
    ConvShape s{c.N * c.To, c.C, c.H, c.W, c.K, c.kh, c.kw, c.d, c.Ho, c.Wo};
    if (c.kt > 1) {
        s.bgroup = c.To;
        s.bskip = c.T - c.To;
        s.in_extent = (long)c.N * c.T * c.frame_in() - (long)e * c.dt * c.frame_in();
    }
    return s;
}

// Backward-data of the frames [t0, t0 + cnt) of one video, all of which reach the same temporal taps e_lo..e_hi:
// the contraction runs over (tap, filter) in the order of increasing source frame, i.e. reversed taps r = kt-1-e.
struct BwdDataCall {
    ConvShape s;
    long dy_frame;      // first source frame (of the video) = t0 - e_hi*dt
    int r_lo;           // first reversed tap
    int t0, cnt;
};

BwdDataCall bwd_data_call(const Conv3 &c, int t0, int cnt, int e_lo, int e_hi)
{
    BwdDataCall q{};
    const int n_e = e_hi - e_lo + 1;
    q.s = ConvShape{cnt, c.C, c.H, c.W, n_e * c.K, c.kh, c.kw, c.d, c.Ho, c.Wo};
    q.dy_frame = (long)t0 - (long)e_hi * c.dt;
    q.r_lo = c.kt - 1 - e_hi;
    q.t0 = t0; q.cnt = cnt;
    if (c.kt > 1) {
        q.s.gsize = c.K;
        q.s.gjump = (long)(c.dt - 1) * c.frame_out();
    }
    return q;
}

// temporal taps frame t of the input reaches: 0 <= t - e*dt < To
inline void tap_range(const Conv3 &c, int t, int &e_lo, int &e_hi)
{
    e_hi = t / c.dt < c.kt - 1 ? t / c.dt : c.kt - 1;
    const int over = t - c.To + 1;      // t - e*dt <= To - 1
    e_lo = over <= 0 ? 0 : (over + c.dt - 1) / c.dt;
}

// calls for one video: one per run of consecutive frames that reach the same temporal taps (kt = 2, dt = 4: the
// first four frames see tap 0 only, the last four tap 1 only, those between both); visit(call) or visit_zero(t0, cnt)
template <typename F, typename Z>
int for_bwd_data_calls(const Conv3 &c, F &&visit, Z &&visit_zero)
{
    for (int t = 0; t < c.T;) {
        int e_lo, e_hi;
        tap_range(c, t, e_lo, e_hi);
        int t1 = t + 1;
        for (; t1 < c.T; ++t1) {
            int lo, hi;
            tap_range(c, t1, lo, hi);
            if (lo != e_lo || hi != e_hi) break;
        }
        const int rc = e_lo > e_hi ? visit_zero(t, t1 - t) : visit(bwd_data_call(c, t, t1 - t, e_lo, e_hi));
        if (rc != DSK_OK) return rc;
        t = t1;
    }
    return DSK_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad_ptr(const void *p) { return p == nullptr || !aligned16(p); }
inline bool bad_dtype(int t) { return t != DSK_F32 && t != DSK_BF16; }
constexpr long kMaxElems = 0x7fffffffL;

int conv3_shape(int N, int T, int C, int H, int W, int K, int kt, int kh, int kw, int dt, int d, Conv3 *c)
{
    if (N < 1 || T < 1 || C < 1 || H < 1 || W < 1 || K < 1 || kt < 1 || kh < 1 || kw < 1 || dt < 1 || d < 1) return DSK_EINVAL;
    const long To = (long)T - (long)(kt - 1) * dt, Ho = (long)H - (long)(kh - 1) * d, Wo = (long)W - (long)(kw - 1) * d;
    if (To < 1 || Ho < 1 || Wo < 1) return DSK_ESHAPE;
    if ((long)N * T > kMaxElems / ((long)C * H * W) || (long)N * To > kMaxElems / ((long)K * Ho * Wo) ||
        (long)kt * K > kMaxElems / ((long)C * kh * kw) || (long)kt * C > (1 << 20) || (long)kt * K > (1 << 20))
        return DSK_ESHAPE;
    *c = Conv3{N, T, C, H, W, K, kt, kh, kw, dt, d, (int)To, (int)Ho, (int)Wo};
    return DSK_OK;
}

size_t conv3_ws_bytes(int which, const Conv3 &c, dsk_dtype in)
{
    if (which == DSK_WS_CONV_FWD)
        return (c.kt > 1 ? align256(4 * (size_t)c.kt * c.w2d()) : 0) + conv_ws_bytes(which, fwd_shape(c), in);
    if (which == DSK_WS_CONV_BWD_WEIGHT) {
        size_t m = 0;
        for (int e = 0; e < c.kt; ++e) {
            const size_t b = conv_ws_bytes(which, bww_shape(c, e), in);
            m = b > m ? b : m;
        }
        return m;
    }
    if (which == DSK_WS_CONV_BWD_DATA) {
        size_t m = 0;
        for_bwd_data_calls(c, [&](const BwdDataCall &q) {
            const size_t b = conv_ws_bytes(which, q.s, in);
            m = b > m ? b : m;
            return (int)DSK_OK; }, [](int, int) { return (int)DSK_OK; });
        return (c.kt > 1 ? align256(4 * (size_t)c.kt * c.w2d()) : 0) + m;
    }
    return 0;
}

// ---------------------------------------------------------------------------------------------------------
// 3-D pooling.  A thread owns four neighbouring columns of one row of one output plane; every tap is one
// 16-byte (bf16: 8-byte) access at any alignment.  The taps of a window are re-read from the caches, HBM sees
// every input element once.  Groups that are cut by the end of a row are taken element by element (a wide
// access reaching past the end of the tensor would lose the elements next to it to the buffer's range check).
// Ties: taps are visited in the order (e*k + a)*k + b and replace the maximum only when strictly greater.
// ---------------------------------------------------------------------------------------------------------
struct Pool3 {
    int N, T, C, H, W, kt, k, dt, d, To, Ho, Wo;
    int groups, bpp;       // column groups per row; workgroups per plane
    long in_elems, out_elems;
};

typedef float pf4 __attribute__((ext_vector_type(4)));
typedef unsigned pu4 __attribute__((ext_vector_type(4)));
typedef unsigned pu2 __attribute__((ext_vector_type(2)));

__device__ inline void ld4(BufRsrc r, const float *, unsigned off, float (&o)[4])
{
    const pf4 t = __builtin_bit_cast(pf4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(off * 4u), 0, 0));
    o[0] = t[0]; o[1] = t[1]; o[2] = t[2]; o[3] = t[3];
}
__device__ inline void ld4(BufRsrc r, const bf16 *, unsigned off, float (&o)[4])
{
    const pu2 t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)(off * 2u), 0, 0);
    o[0] = __builtin_bit_cast(float, t[0] << 16); o[1] = __builtin_bit_cast(float, t[0] & 0xffff0000u);
    o[2] = __builtin_bit_cast(float, t[1] << 16); o[3] = __builtin_bit_cast(float, t[1] & 0xffff0000u);
}
__device__ inline void st4(BufRsrc r, float *, unsigned off, const float (&v)[4])
{
    const pf4 t = {v[0], v[1], v[2], v[3]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(pu4, t), r, (int)(off * 4u), 0, 0);
}
__device__ inline void st4(BufRsrc r, bf16 *, unsigned off, const float (&v)[4])
{
    const pu2 t = {(unsigned)f32_to_bf16(v[0]).v | (unsigned)f32_to_bf16(v[1]).v << 16,
                   (unsigned)f32_to_bf16(v[2]).v | (unsigned)f32_to_bf16(v[3]).v << 16};
    __builtin_amdgcn_raw_buffer_store_b64(t, r, (int)(off * 2u), 0, 0);
}

// KT, K: window sizes known at compile time (0: taken from s); then all taps of a thread are loaded before the
// first is used, instead of one memory round trip per tap.
template <typename T, bool IS_MAX, int KT, int K>
__global__ void __launch_bounds__(kThreads)
pool3d_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, Pool3 s)
{
    const int kt = KT ? KT : s.kt, k = K ? K : s.k;
    const int op = (int)(blockIdx.x / (unsigned)s.bpp);      // output plane (n*To + t)*C + c
    const int tt = (int)(blockIdx.x % (unsigned)s.bpp) * kThreads + (int)threadIdx.x;
    const int row = tt / s.groups, col = (tt - row * s.groups) * 4;
    if (row >= s.Ho) return;
    const int c = op % s.C, ft = op / s.C, n = ft / s.To, t = ft - n * s.To;
    const unsigned HW = (unsigned)(s.H * s.W), HoWo = (unsigned)(s.Ho * s.Wo);
    const T *xp = x + ((long)(n * s.T + t) * s.C + c) * HW;      // tap e = 0
    T *yp = y + (long)op * HoWo;
    const BufRsrc rx = buf_rsrc(xp, x + s.in_elems), ry = buf_rsrc(yp, y + s.out_elems);
    const unsigned fstride = (unsigned)(s.dt * s.C) * HW;      // elements between temporal taps (the host bounds kt*fstride)
    const int nv = s.Wo - col < 4 ? s.Wo - col : 4;
    float best[4] = {0.f, 0.f, 0.f, 0.f};
    int bi[4] = {0, 0, 0, 0};
    auto visit = [&](int tap, const float (&v)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (IS_MAX) {
                if (tap == 0 || v[j] > best[j]) { best[j] = v[j]; bi[j] = tap; }
            } else {
                best[j] += v[j];
            }
        }
    };
    if (KT != 0 && nv == 4) {
        float v[(KT ? KT * K * K : 1)][4];
#pragma unroll
        for (int e = 0; e < KT; ++e)
#pragma unroll
            for (int a = 0; a < K; ++a)
#pragma unroll
                for (int b = 0; b < K; ++b)
                    ld4(rx, xp, (unsigned)e * fstride + (unsigned)((row + a * s.d) * s.W + col + b * s.d), v[(e * K + a) * K + b]);
#pragma unroll
        for (int t = 0; t < KT * K * K; ++t) visit(t, v[t]);
    } else {
        int tap = 0;
        for (int e = 0; e < kt; ++e)
            for (int a = 0; a < k; ++a)
                for (int b = 0; b < k; ++b, ++tap) {
                    const unsigned off = (unsigned)e * fstride + (unsigned)((row + a * s.d) * s.W + col + b * s.d);
                    float v[4] = {0.f, 0.f, 0.f, 0.f};
                    if (nv == 4) {
                        ld4(rx, xp, off, v);
                    } else {
                        for (int j = 0; j < nv; ++j) v[j] = buf_ld(rx, xp, off + (unsigned)j, 0u);
                    }
                    visit(tap, v);
                }
    }
    if (!IS_MAX) {
        const float inv = 1.f / (float)(kt * k * k);
#pragma unroll
        for (int j = 0; j < 4; ++j) best[j] *= inv;
    }
    const unsigned oo = (unsigned)(row * s.Wo + col);
    if (nv == 4) {
        st4(ry, yp, oo, best);
    } else {
        for (int j = 0; j < nv; ++j) buf_st(ry, yp, oo + (unsigned)j, 0u, best[j]);
    }
    if (IS_MAX && am) {
        uint8_t *ap = am + (long)op * HoWo;
        const BufRsrc ra = buf_rsrc(ap, am + s.out_elems);
        if (nv == 4) {
            __builtin_amdgcn_raw_buffer_store_b32((unsigned)bi[0] | (unsigned)bi[1] << 8 | (unsigned)bi[2] << 16 | (unsigned)bi[3] << 24,
                                                  ra, (int)oo, 0, 0);
        } else {
            for (int j = 0; j < nv; ++j) buf_st(ra, ap, oo + (unsigned)j, 0u, bi[j]);
        }
    }
}

// Gather form: every input element adds up the outputs whose window holds it (and, for max pooling, whose
// recorded winner it is); fixed order, no atomics.
// KT, K as in the forward kernel: with compile-time sizes the candidate outputs of all taps are loaded together
// (from a harmless address where a tap does not apply), then added in a fixed order.
template <typename T, bool IS_MAX, int KT, int K>
__global__ void __launch_bounds__(kThreads)
pool3d_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, Pool3 s)
{
    const int ip = (int)(blockIdx.x / (unsigned)s.bpp);      // input plane (n*T + t)*C + c
    const int tt = (int)(blockIdx.x % (unsigned)s.bpp) * kThreads + (int)threadIdx.x;
    const int row = tt / s.groups, col = (tt - row * s.groups) * 4;
    if (row >= s.H) return;
    const int c = ip % s.C, ft = ip / s.C, n = ft / s.T, t = ft - n * s.T;
    // temporal taps this frame is reached by: 0 <= t - e*dt < To
    int e_hi = t / s.dt < s.kt - 1 ? t / s.dt : s.kt - 1;
    const int over = t - s.To + 1;
    const int e_lo = over <= 0 ? 0 : (over + s.dt - 1) / s.dt;
    const unsigned HW = (unsigned)(s.H * s.W), HoWo = (unsigned)(s.Ho * s.Wo);
    T *dxp = dx + (long)ip * HW;
    const BufRsrc rdx = buf_rsrc(dxp, dx + s.in_elems);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (e_lo <= e_hi) {
        // the earliest source frame first: offsets from it are never negative
        const long p0 = ((long)(n * s.To + t - e_hi * s.dt) * s.C + c) * HoWo;
        const T *dyp = dy + p0;
        const uint8_t *ap = IS_MAX ? am + p0 : nullptr;
        const BufRsrc rdy = buf_rsrc(dyp, dy + s.out_elems);
        const BufRsrc ra = buf_rsrc(ap, IS_MAX ? am + s.out_elems : ap);
        const unsigned fstride = (unsigned)(s.dt * s.C) * HoWo;
        // one tap, element by element (groups cut by the ends of a row)
        auto tap_by_element = [&](int e, int a, int b) __attribute__((always_inline)) {
            const int u = row - a * s.d, v0 = col - b * s.d;
            const int tap = (e * s.k + a) * s.k + b;
            const unsigned fo = (unsigned)(e_hi - e) * fstride;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int v = v0 + j;
                if (v < 0 || v >= s.Wo) continue;
                const unsigned o = fo + (unsigned)(u * s.Wo + v);
                const float g = buf_ld(rdy, dyp, o, 0u);
                if (IS_MAX) acc[j] += buf_ld(ra, ap, o, 0u) == tap ? g : 0.f;
                else acc[j] += g;
            }
        };
        if (KT != 0) {
            constexpr int NT = KT ? KT * K * K : 1;
            float g[NT][4];
            unsigned w[NT];
            unsigned full = 0, part = 0;      // bit t: all four / some of the four candidate outputs of tap t exist
#pragma unroll
            for (int e = 0; e < KT; ++e)
#pragma unroll
                for (int a = 0; a < K; ++a)
#pragma unroll
                    for (int b = 0; b < K; ++b) {
                        const int t = (e * K + a) * K + b;
                        const int u = row - a * s.d, v0 = col - b * s.d;
                        const bool here = e >= e_lo && e <= e_hi && u >= 0 && u < s.Ho;
                        const bool all4 = here && v0 >= 0 && v0 + 3 < s.Wo;
                        full |= all4 ? 1u << t : 0u;
                        part |= here && !all4 && v0 + 3 >= 0 && v0 < s.Wo ? 1u << t : 0u;
                        const unsigned off = all4 ? (unsigned)(e_hi - e) * fstride + (unsigned)(u * s.Wo + v0) : 0u;
                        ld4(rdy, dyp, off, g[t]);
                        w[t] = IS_MAX ? (unsigned)__builtin_amdgcn_raw_buffer_load_b32(ra, (int)off, 0, 0) : 0u;
                    }
#pragma unroll
            for (int t = NT - 1; t >= 0; --t) {
                if ((full >> t) & 1u) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] += !IS_MAX || (int)((w[t] >> (8 * j)) & 0xffu) == t ? g[t][j] : 0.f;
                } else if ((part >> t) & 1u) {
                    tap_by_element(t / (K * K), (t / K) % K, t % K);
                }
            }
        } else
        for (int e = e_hi; e >= e_lo; --e) {
            const unsigned fo = (unsigned)(e_hi - e) * fstride;
            for (int a = 0; a < s.k; ++a) {
                const int u = row - a * s.d;
                if (u < 0 || u >= s.Ho) continue;
                for (int b = 0; b < s.k; ++b) {
                    const int v0 = col - b * s.d;
                    const int tap = (e * s.k + a) * s.k + b;
                    const unsigned off = fo + (unsigned)(u * s.Wo + v0);      // meaningless where v0 < 0: not used then
                    if (v0 >= 0 && v0 + 3 < s.Wo) {
                        float g[4];
                        ld4(rdy, dyp, off, g);
                        if (IS_MAX) {
                            const unsigned w = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(ra, (int)off, 0, 0);
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[j] += (int)((w >> (8 * j)) & 0xffu) == tap ? g[j] : 0.f;
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[j] += g[j];
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int v = v0 + j;
                            if (v < 0 || v >= s.Wo) continue;
                            const unsigned o = fo + (unsigned)(u * s.Wo + v);
                            const float g = buf_ld(rdy, dyp, o, 0u);
                            if (IS_MAX) acc[j] += buf_ld(ra, ap, o, 0u) == tap ? g : 0.f;
                            else acc[j] += g;
                        }
                    }
                }
            }
        }
    }
    if (!IS_MAX) {
        const float inv = 1.f / (float)(s.kt * s.k * s.k);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] *= inv;
    }
    const int nv = s.W - col < 4 ? s.W - col : 4;
    const unsigned oo = (unsigned)(row * s.W + col);
    if (nv == 4) {
        st4(rdx, dxp, oo, acc);
    } else {
        for (int j = 0; j < nv; ++j) buf_st(rdx, dxp, oo + (unsigned)j, 0u, acc[j]);
    }
}

int pool3_shape(const void *a, const void *b, int N, int T, int C, int H, int W, int kt, int k, int dt, int d, int t, Pool3 *p)
{
    if (bad_ptr(a) || bad_ptr(b) || bad_dtype(t)) return DSK_EINVAL;
    if (N < 1 || T < 1 || C < 1 || H < 1 || W < 1 || kt < 1 || k < 1 || dt < 1 || d < 1) return DSK_EINVAL;
    if ((long)kt * k * k > 255) return DSK_ESHAPE;
    const long To = (long)T - (long)(kt - 1) * dt, Ho = (long)H - (long)(k - 1) * d, Wo = (long)W - (long)(k - 1) * d;
    if (To < 1 || Ho < 1 || Wo < 1) return DSK_ESHAPE;
    if ((long)N * T > kMaxElems / ((long)C * H * W)) return DSK_ESHAPE;
    // 32-bit element offsets from the plane of the first temporal tap
    if ((long)kt * dt * C * H * W >= (1L << 30)) return DSK_ESHAPE;
    *p = Pool3{N, T, C, H, W, kt, k, dt, d, (int)To, (int)Ho, (int)Wo, 0, 0,
               (long)N * T * C * H * W, (long)N * To * C * Ho * Wo};
    return DSK_OK;
}

template <bool IS_MAX>
int pool3_fwd(const void *x, void *y, uint8_t *am, Pool3 p, dsk_dtype t, hipStream_t st)
{
    p.groups = (p.Wo + 3) / 4;
    p.bpp = (int)(((long)p.Ho * p.groups + kThreads - 1) / kThreads);
    const long blocks = (long)p.N * p.To * p.C * p.bpp;
    if (blocks > 0x7fffffffL) return DSK_ESHAPE;
    clear_errors();
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (p.kt == 2 && p.k == 2) {
        if (t == DSK_F32) pool3d_fwd_kernel<float, IS_MAX, 2, 2><<<grid, block, 0, st>>>((const float *)x, (float *)y, am, p);
        else pool3d_fwd_kernel<bf16, IS_MAX, 2, 2><<<grid, block, 0, st>>>((const bf16 *)x, (bf16 *)y, am, p);
    } else {
        if (t == DSK_F32) pool3d_fwd_kernel<float, IS_MAX, 0, 0><<<grid, block, 0, st>>>((const float *)x, (float *)y, am, p);
        else pool3d_fwd_kernel<bf16, IS_MAX, 0, 0><<<grid, block, 0, st>>>((const bf16 *)x, (bf16 *)y, am, p);
    }
    return check_launch();
}

template <bool IS_MAX>
int pool3_bwd(const void *dy, const uint8_t *am, void *dx, Pool3 p, dsk_dtype t, hipStream_t st)
{
    p.groups = (p.W + 3) / 4;
    p.bpp = (int)(((long)p.H * p.groups + kThreads - 1) / kThreads);
    const long blocks = (long)p.N * p.T * p.C * p.bpp;
    if (blocks > 0x7fffffffL) return DSK_ESHAPE;
    clear_errors();
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (p.kt == 2 && p.k == 2) {
        if (t == DSK_F32) pool3d_bwd_kernel<float, IS_MAX, 2, 2><<<grid, block, 0, st>>>((const float *)dy, am, (float *)dx, p);
        else pool3d_bwd_kernel<bf16, IS_MAX, 2, 2><<<grid, block, 0, st>>>((const bf16 *)dy, am, (bf16 *)dx, p);
    } else {
        if (t == DSK_F32) pool3d_bwd_kernel<float, IS_MAX, 0, 0><<<grid, block, 0, st>>>((const float *)dy, am, (float *)dx, p);
        else pool3d_bwd_kernel<bf16, IS_MAX, 0, 0><<<grid, block, 0, st>>>((const bf16 *)dy, am, (bf16 *)dx, p);
    }
    return check_launch();
}

} // namespace

} // namespace dsk

using namespace dsk;

extern "C" {

size_t dsk_conv3d_workspace_bytes(int which, int N, int T, int C, int H, int W, int K, int kt, int kh, int kw, int dt,
                                  int d, dsk_dtype in)
{
    Conv3 c;
    if (conv3_shape(N, T, C, H, W, K, kt, kh, kw, dt, d, &c) != DSK_OK || bad_dtype(in)) return 0;
    return conv3_ws_bytes(which, c, in);
}

int dsk_conv3d_fwd(const void *x, const float *w, const float *b, void *y, int N, int T, int C, int H, int W, int K,
                   int kt, int kh, int kw, int dt, int d, dsk_dtype in, dsk_dtype out, dsk_act act, void *ws,
                   size_t ws_bytes, void *stream)
{
    if (bad_ptr(x) || bad_ptr(w) || bad_ptr(y) || (b && !aligned16(b))) return DSK_EINVAL;
    if (bad_dtype(in) || bad_dtype(out) || act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    Conv3 c;
    const int rc = conv3_shape(N, T, C, H, W, K, kt, kh, kw, dt, d, &c);
    if (rc != DSK_OK) return rc;
    const size_t need = conv3_ws_bytes(DSK_WS_CONV_FWD, c, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    clear_errors();
    const float *w2 = w;
    void *ws2 = ws;
    if (c.kt > 1) {
        const long total = (long)c.kt * c.w2d();
        w3_forward_order_kernel<<<dim3(blocks_for(total)), dim3(kThreads), 0, st>>>(w, (float *)ws, c.kt, c.K, c.C, (int)c.taps());
        if (check_launch() != DSK_OK) return DSK_ELAUNCH;
        w2 = (const float *)ws;
        ws2 = (char *)ws + align256(4 * (size_t)total);
    }
    return dispatch_conv_fwd(x, w2, b, y, fwd_shape(c), in, out, act, ws2, st);
}

int dsk_conv3d_bwd_data(const void *dy, const float *w, void *dx, int N, int T, int C, int H, int W, int K, int kt,
                        int kh, int kw, int dt, int d, dsk_dtype in, dsk_dtype out, void *ws, size_t ws_bytes,
                        void *stream)
{
    if (bad_ptr(dy) || bad_ptr(w) || bad_ptr(dx) || bad_dtype(in) || bad_dtype(out)) return DSK_EINVAL;
    Conv3 c;
    int rc = conv3_shape(N, T, C, H, W, K, kt, kh, kw, dt, d, &c);
    if (rc != DSK_OK) return rc;
    const size_t need = conv3_ws_bytes(DSK_WS_CONV_BWD_DATA, c, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    clear_errors();
    const float *wr = w;
    void *ws2 = ws;
    if (c.kt > 1) {
        const long total = (long)c.kt * c.w2d();
        w3_reverse_kernel<<<dim3(blocks_for(total)), dim3(kThreads), 0, st>>>(w, (float *)ws, c.kt, c.w2d());
        if (check_launch() != DSK_OK) return DSK_ELAUNCH;
        wr = (const float *)ws;
        ws2 = (char *)ws + align256(4 * (size_t)total);
    }
    const size_t ein = in == DSK_F32 ? 4 : 2, eout = out == DSK_F32 ? 4 : 2;
    const long dy_total = (long)c.N * c.To * c.frame_out();
    for (int n = 0; n < c.N; ++n) {
        rc = for_bwd_data_calls(c,
            [&](BwdDataCall q) {
                const long first = ((long)n * c.To + q.dy_frame) * c.frame_out();      // elements into dy
                q.s.in_extent = dy_total - first;
                return dispatch_conv_bwd_data((const char *)dy + first * ein, wr + (long)q.r_lo * c.w2d(),
                                              (char *)dx + ((long)n * c.T + q.t0) * c.frame_in() * eout, q.s, in, out, ws2, st);
            },
            [&](int t, int cnt) {
                // frames no output frame looks at (fewer output frames than the temporal spacing)
                void *p = (char *)dx + ((long)n * c.T + t) * c.frame_in() * eout;
                const long count = (long)cnt * c.frame_in();
                if (out == DSK_F32) fill_zero_kernel<float><<<dim3(blocks_for(count)), dim3(kThreads), 0, st>>>((float *)p, count);
                else fill_zero_kernel<bf16><<<dim3(blocks_for(count)), dim3(kThreads), 0, st>>>((bf16 *)p, count);
                return check_launch();
            });
        if (rc != DSK_OK) return rc;
    }
    return DSK_OK;
}

int dsk_conv3d_bwd_weight(const void *x, const void *dy, float *dw, float *db, int N, int T, int C, int H, int W,
                          int K, int kt, int kh, int kw, int dt, int d, dsk_dtype in, void *ws, size_t ws_bytes,
                          void *stream)
{
    if (bad_ptr(x) || bad_ptr(dy) || bad_ptr(dw) || (db && !aligned16(db)) || bad_dtype(in)) return DSK_EINVAL;
    Conv3 c;
    int rc = conv3_shape(N, T, C, H, W, K, kt, kh, kw, dt, d, &c);
    if (rc != DSK_OK) return rc;
    const size_t need = conv3_ws_bytes(DSK_WS_CONV_BWD_WEIGHT, c, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    clear_errors();
    const size_t ein = in == DSK_F32 ? 4 : 2;
    for (int e = 0; e < c.kt; ++e) {
        rc = dispatch_conv_bwd_weight((const char *)x + (long)e * c.dt * c.frame_in() * ein, dy, dw + (long)e * c.w2d(),
                                      e == 0 ? db : nullptr, bww_shape(c, e), in, ws, st);
        if (rc != DSK_OK) return rc;
    }
    return DSK_OK;
}

int dsk_pad_video(const float *x, void *xpad, int N, int T, int C, int H, int W, int tlo, int thi, int lo, int hi,
                  dsk_dtype out, void *stream)
{
    if (bad_ptr(x) || bad_ptr(xpad) || bad_dtype(out)) return DSK_EINVAL;
    if (N < 1 || T < 1 || C < 1 || H < 1 || W < 1 || tlo < 0 || thi < 0 || lo < 0 || hi < 0) return DSK_EINVAL;
    const long Tp = (long)T + tlo + thi, Hp = (long)H + lo + hi, Wp = (long)W + lo + hi;
    if (Tp > kMaxElems || Hp > kMaxElems || Wp > kMaxElems || (long)N * Tp > kMaxElems / ((long)C * Hp * Wp)) return DSK_ESHAPE;
    const long total = (long)N * Tp * C * Hp * Wp;
    clear_errors();
    if (out == DSK_F32)
        pad_video_kernel<float><<<dim3(blocks_for(total)), dim3(kThreads), 0, (hipStream_t)stream>>>(
            x, (float *)xpad, N, T, C, H, W, tlo, lo, (int)Tp, (int)Hp, (int)Wp);
    else
        pad_video_kernel<bf16><<<dim3(blocks_for(total)), dim3(kThreads), 0, (hipStream_t)stream>>>(
            x, (bf16 *)xpad, N, T, C, H, W, tlo, lo, (int)Tp, (int)Hp, (int)Wp);
    return check_launch();
}

int dsk_maxpool3d_fwd(const void *x, void *y, uint8_t *argmax, int N, int T, int C, int H, int W, int kt, int k, int dt,
                      int d, dsk_dtype t, void *stream)
{
    Pool3 p;
    const int rc = pool3_shape(x, y, N, T, C, H, W, kt, k, dt, d, t, &p);
    if (rc != DSK_OK) return rc;
    if (argmax && !aligned16(argmax)) return DSK_EINVAL;
    return pool3_fwd<true>(x, y, argmax, p, t, (hipStream_t)stream);
}

int dsk_maxpool3d_bwd(const void *dy, const uint8_t *argmax, void *dx, int N, int T, int C, int H, int W, int kt, int k,
                      int dt, int d, dsk_dtype t, void *stream)
{
    Pool3 p;
    const int rc = pool3_shape(dy, dx, N, T, C, H, W, kt, k, dt, d, t, &p);
    if (rc != DSK_OK) return rc;
    if (bad_ptr(argmax)) return DSK_EINVAL;
    return pool3_bwd<true>(dy, argmax, dx, p, t, (hipStream_t)stream);
}

int dsk_avgpool3d_fwd(const void *x, void *y, int N, int T, int C, int H, int W, int kt, int k, int dt, int d,
                      dsk_dtype t, void *stream)
{
    Pool3 p;
    const int rc = pool3_shape(x, y, N, T, C, H, W, kt, k, dt, d, t, &p);
    if (rc != DSK_OK) return rc;
    return pool3_fwd<false>(x, y, nullptr, p, t, (hipStream_t)stream);
}

int dsk_avgpool3d_bwd(const void *dy, void *dx, int N, int T, int C, int H, int W, int kt, int k, int dt, int d,
                      dsk_dtype t, void *stream)
{
    Pool3 p;
    const int rc = pool3_shape(dy, dx, N, T, C, H, W, kt, k, dt, d, t, &p);
    if (rc != DSK_OK) return rc;
    return pool3_bwd<false>(dy, nullptr, dx, p, t, (hipStream_t)stream);
}

} // extern "C"
