// Stride-1 pooling with d-regularly sparse k x k kernels (paper Sec. 3.1-3.2;
// backward Sec. 4.2).  Bandwidth-bound: every input element should come from
// HBM once.  A thread owns one column and R output rows that lie in ONE residue
// class modulo d (rows u0, u0+d, u0+2d, ...): the k taps of neighbouring outputs
// in that class share input rows, so R outputs need R+k-1 row visits instead of
// R*k, and every wavefront load is one contiguous row segment.  Column taps
// (v, v+d, ...) of a wavefront overlap in the same cache lines.
//
// Max-pool ties: taps are ranked by a*k+b and only a strictly greater value
// replaces the running maximum, so the lowest index wins.  Taking the first
// maximum of each input row and then the first row holding the overall maximum
// selects exactly that tap.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kPoolThreads = 256;

struct PoolShape {
    int planes, H, W, Ho, Wo, k, d;
    int col_blocks, row_groups;   // row_groups = ceil(rows / (d*R)) * d
};

// Decode blockIdx.x -> (plane, first row of the residue class, column).
template <int R>
__device__ inline void pool_decode(const PoolShape &s, int rows, int &plane, int &r0, int &col)
{
    long b = blockIdx.x;
    const int cb = (int)(b % s.col_blocks);
    b /= s.col_blocks;
    const int rg = (int)(b % s.row_groups);
    plane = (int)(b / s.row_groups);
    const int grp = rg / s.d, res = rg % s.d;
    r0 = grp * s.d * R + res;
    col = cb * kPoolThreads + threadIdx.x;
    (void)rows;
}

// All loads of a thread are issued before anything depends on one of them: rows and columns
// that do not exist are clamped to ones that do (their values are never used), so no load sits
// under a condition, and every access is a buffer access with one per-lane offset per tap
// column and a scalar offset per row.
template <typename T, int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    int plane, u0, v;
    pool_decode<R>(s, s.Ho, plane, u0, v);
    if (u0 >= s.Ho) return;
    const bool col_ok = v < s.Wo;
    unsigned vc = col_ok ? (unsigned)v : 0u;      // column 0 exists; v + b*d < W whenever v < Wo
    const T *xp = x + (long)plane * s.H * s.W;
    const BufRsrc rx = buf_rsrc(xp, xp + (long)s.H * s.W);
    // rows per batch of loads: all of them for small windows; one row (K loads) for large ones,
    // which would otherwise need (R+K-1)*K registers
    constexpr int NT = R + K - 1, TB = K <= 3 ? NT : 1;
    float rowv[NT];
    int rowi[NT];
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += TB) {
        float xv[TB][K];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            int row = u0 + (t0 + t) * s.d;
            row = row < s.H ? row : s.H - 1;
#pragma unroll
            for (int b = 0; b < K; ++b) xv[t][b] = buf_ld(rx, xp, vc + (unsigned)(b * s.d), (unsigned)(row * s.W));
        }
        // the values are pinned here so that the loads of a batch are issued together above,
        // not one by one where the branches below use them
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int b = 0; b < K; ++b) asm volatile("" : "+v"(xv[t][b]));
        // ... and the next batch is not hoisted above this one (its offset "changes" here)
        if (TB < NT) asm volatile("" : "+v"(vc));
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            float best = xv[t][0];
            int bi = 0;
#pragma unroll
            for (int b = 1; b < K; ++b) {
                if (IS_MAX) {
                    if (xv[t][b] > best) { best = xv[t][b]; bi = b; }
                } else {
                    best += xv[t][b];
                }
            }
            rowv[t0 + t] = best;
            rowi[t0 + t] = bi;
        }
    }
    if (!col_ok) return;
    T *yp = y + (long)plane * s.Ho * s.Wo;
    const BufRsrc ry = buf_rsrc(yp, yp + (long)s.Ho * s.Wo);
    uint8_t *ap = IS_MAX && am ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc ra = buf_rsrc(ap, ap + (ap ? (long)s.Ho * s.Wo : 0));
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int u = u0 + r * s.d;
        if (u >= s.Ho) break;
        float best = rowv[r];
        int bi = rowi[r];
        if (IS_MAX) {
#pragma unroll
            for (int a = 1; a < K; ++a)
                if (rowv[r + a] > best) { best = rowv[r + a]; bi = a * K + rowi[r + a]; }
        } else {
#pragma unroll
            for (int a = 1; a < K; ++a) best += rowv[r + a];
            best *= 1.0f / (float)(K * K);
        }
        buf_st(ry, yp, (unsigned)v, (unsigned)(u * s.Wo), best);
        if (ap) buf_st(ra, ap, (unsigned)v, (unsigned)(u * s.Wo), bi);
    }
}

// dx rows p0 + r*d (r < R) of one column: they collect from dy rows p0 + (r-a)*d.
template <typename T, int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, PoolShape s)
{
    int plane, p0, q;
    pool_decode<R>(s, s.H, plane, p0, q);
    if (p0 >= s.H) return;
    const bool col_ok = q < s.W;
    const T *dyp = dy + (long)plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc rg = buf_rsrc(dyp, dyp + (long)s.Ho * s.Wo);
    const BufRsrc ra = buf_rsrc(amp, amp + (IS_MAX ? (long)s.Ho * s.Wo : 0));
    // dy column q - b*d, clamped into the map; `cok` bit b says that it exists
    unsigned vcol[K];
    unsigned cok = 0;
#pragma unroll
    for (int b = 0; b < K; ++b) {
        const int v = q - b * s.d;
        const bool ok = col_ok && v >= 0 && v < s.Wo;
        vcol[b] = ok ? (unsigned)v : 0u;
        cok |= ok ? 1u << b : 0u;
    }
    // t indexes dy rows p0 + (t-(K-1))*d, t = 0 .. R+K-2; it feeds dx rows r = t-(K-1)+a.
    // Rows per batch of loads: all of them for small windows, one row (2K loads) for large ones.
    constexpr int NT = R + K - 1, TB = K <= 3 ? NT : 1;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += TB) {
        float g[TB][K];
        int idx[TB][K];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            int u = p0 + (t0 + t - (K - 1)) * s.d;
            u = u < 0 ? 0 : (u >= s.Ho ? s.Ho - 1 : u);
#pragma unroll
            for (int b = 0; b < K; ++b) {
                g[t][b] = buf_ld(rg, dyp, vcol[b], (unsigned)(u * s.Wo));
                idx[t][b] = IS_MAX ? buf_ld(ra, amp, vcol[b], (unsigned)(u * s.Wo)) : 0;
            }
        }
        // the values are pinned here so that the loads of a batch are issued together above,
        // not one by one where the branches below use them
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int b = 0; b < K; ++b) {
                asm volatile("" : "+v"(g[t][b]));
                if (IS_MAX) asm volatile("" : "+v"(idx[t][b]));
            }
        // ... and the next batch is not hoisted above this one (its offsets "change" here):
        // one batch in flight per wave keeps the register count, and with it the occupancy, sane
        if (TB < NT)
#pragma unroll
            for (int b = 0; b < K; ++b) asm volatile("" : "+v"(vcol[b]));
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const int u = p0 + (t0 + t - (K - 1)) * s.d;
            const bool row_ok = u >= 0 && u < s.Ho;       // uniform
#pragma unroll
            for (int b = 0; b < K; ++b) {
                const float gv = row_ok && ((cok >> b) & 1u) ? g[t][b] : 0.f;
#pragma unroll
                for (int a = 0; a < K; ++a) {
                    const int r = t0 + t - (K - 1) + a;
                    if (r >= 0 && r < R) acc[r] += !IS_MAX || idx[t][b] == a * K + b ? gv : 0.f;
                }
            }
        }
    }
    if (!col_ok) return;
    T *dxp = dx + (long)plane * s.H * s.W;
    const BufRsrc rd = buf_rsrc(dxp, dxp + (long)s.H * s.W);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = p0 + r * s.d;
        if (p >= s.H) break;
        const float v = IS_MAX ? acc[r] : acc[r] * (1.0f / (float)(K * K));
        buf_st(rd, dxp, (unsigned)q, (unsigned)(p * s.W), v);
    }
}

// ---- any k: one thread per output entry ----
template <typename T, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_fwd_generic_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    const long total = (long)s.planes * s.Ho * s.Wo;
    const long idx = (long)blockIdx.x * kPoolThreads + threadIdx.x;
    if (idx >= total) return;
    const int v = (int)(idx % s.Wo);
    const int u = (int)((idx / s.Wo) % s.Ho);
    const long plane = idx / ((long)s.Wo * s.Ho);
    const T *xp = x + (plane * s.H + u) * s.W + v;
    float best = ldf(xp, 0);
    int bi = 0;
    for (int a = 0; a < s.k; ++a)
        for (int b = 0; b < s.k; ++b) {
            if (a == 0 && b == 0) continue;
            const float t = ldf(xp, (long)a * s.d * s.W + b * s.d);
            if (IS_MAX) {
                if (t > best) { best = t; bi = a * s.k + b; }
            } else {
                best += t;
            }
        }
    if (!IS_MAX) best *= 1.0f / (float)(s.k * s.k);
    stf(y, idx, best);
    if (IS_MAX && am) am[idx] = (uint8_t)bi;
}

template <typename T, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_bwd_generic_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, PoolShape s)
{
    const long total = (long)s.planes * s.H * s.W;
    const long idx = (long)blockIdx.x * kPoolThreads + threadIdx.x;
    if (idx >= total) return;
    const int q = (int)(idx % s.W);
    const int p = (int)((idx / s.W) % s.H);
    const long plane = idx / ((long)s.W * s.H);
    const T *dyp = dy + plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + plane * s.Ho * s.Wo : nullptr;
    float acc = 0.f;
    for (int a = 0; a < s.k; ++a) {
        const int u = p - a * s.d;
        if (u < 0 || u >= s.Ho) continue;
        for (int b = 0; b < s.k; ++b) {
            const int v = q - b * s.d;
            if (v < 0 || v >= s.Wo) continue;
            const long o = (long)u * s.Wo + v;
            if (IS_MAX) {
                if (amp[o] == a * s.k + b) acc += ldf(dyp, o);
            } else {
                acc += ldf(dyp, o);
            }
        }
    }
    if (!IS_MAX) acc *= 1.0f / (float)(s.k * s.k);
    stf(dx, idx, acc);
}

static PoolShape make_shape(int N, int C, int H, int W, int k, int d, int R, int rows, int cols)
{
    PoolShape s;
    s.planes = N * C;
    s.H = H; s.W = W;
    s.Ho = H - (k - 1) * d; s.Wo = W - (k - 1) * d;
    s.k = k; s.d = d;
    s.col_blocks = (cols + kPoolThreads - 1) / kPoolThreads;
    s.row_groups = ((rows + d * R - 1) / (d * R)) * d;
    return s;
}

template <typename T, bool IS_MAX>
static int pool_fwd_dispatch(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                             hipStream_t st)
{
    constexpr int R = 8;
    PoolShape s = make_shape(N, C, H, W, k, d, R, H - (k - 1) * d, W - (k - 1) * d);
    const long tiled_blocks = (long)s.planes * s.row_groups * s.col_blocks;
    if (k == 2 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 2, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 3 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 3, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 4 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 4, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 8 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 8, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else {
        const long total = (long)s.planes * s.Ho * s.Wo;
        pool_fwd_generic_kernel<T, IS_MAX>
            <<<dim3((unsigned)((total + kPoolThreads - 1) / kPoolThreads)), dim3(kPoolThreads), 0, st>>>(
                (const T *)x, (T *)y, am, s);
    }
    return check_launch();
}

template <typename T, bool IS_MAX>
static int pool_bwd_dispatch(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k,
                             int d, hipStream_t st)
{
    // rows per thread: 8 for small windows; 2 for 4x4 and 8x8 ones, whose k*k tests per row pair
    // otherwise unroll into a kernel that needs every register of the SIMD
    constexpr int R = 8, RL = 2;
    PoolShape s = make_shape(N, C, H, W, k, d, k <= 3 ? R : RL, H, W);
    const long tiled_blocks = (long)s.planes * s.row_groups * s.col_blocks;
    if (k == 2 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 2, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 3 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 3, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 4 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 4, RL, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 8 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 8, RL, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else {
        const long total = (long)s.planes * s.H * s.W;
        pool_bwd_generic_kernel<T, IS_MAX>
            <<<dim3((unsigned)((total + kPoolThreads - 1) / kPoolThreads)), dim3(kPoolThreads), 0, st>>>(
                (const T *)dy, am, (T *)dx, s);
    }
    return check_launch();
}

int launch_maxpool_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st)
{
    return t == DSK_F32 ? pool_fwd_dispatch<float, true>(x, y, am, N, C, H, W, k, d, st)
                        : pool_fwd_dispatch<bf16, true>(x, y, am, N, C, H, W, k, d, st);
}

int launch_maxpool_bwd(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st)
{
    return t == DSK_F32 ? pool_bwd_dispatch<float, true>(dy, am, dx, N, C, H, W, k, d, st)
                        : pool_bwd_dispatch<bf16, true>(dy, am, dx, N, C, H, W, k, d, st);
}

int launch_avgpool_fwd(const void *x, void *y, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st)
{
    return t == DSK_F32 ? pool_fwd_dispatch<float, false>(x, y, nullptr, N, C, H, W, k, d, st)
                        : pool_fwd_dispatch<bf16, false>(x, y, nullptr, N, C, H, W, k, d, st);
}

int launch_avgpool_bwd(const void *dy, void *dx, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st)
{
    return t == DSK_F32 ? pool_bwd_dispatch<float, false>(dy, nullptr, dx, N, C, H, W, k, d, st)
                        : pool_bwd_dispatch<bf16, false>(dy, nullptr, dx, N, C, H, W, k, d, st);
}

} // namespace dsk
