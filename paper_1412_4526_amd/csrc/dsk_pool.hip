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

template <typename T, int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    int plane, u0, v;
    pool_decode<R>(s, s.Ho, plane, u0, v);
    if (v >= s.Wo || u0 >= s.Ho) return;
    const T *xp = x + (long)plane * s.H * s.W;
    float rowv[R + K - 1];
    int rowi[R + K - 1];
#pragma unroll
    for (int t = 0; t < R + K - 1; ++t) {
        const int row = u0 + t * s.d;
        rowv[t] = 0.f;
        rowi[t] = 0;
        if (row < s.H) {
            const T *rp = xp + (long)row * s.W + v;
            float best = ldf(rp, 0);
            int bi = 0;
            if (IS_MAX) {
#pragma unroll
                for (int b = 1; b < K; ++b) {
                    const float tv = ldf(rp, (long)b * s.d);
                    if (tv > best) { best = tv; bi = b; }
                }
            } else {
#pragma unroll
                for (int b = 1; b < K; ++b) best += ldf(rp, (long)b * s.d);
            }
            rowv[t] = best;
            rowi[t] = bi;
        }
    }
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
        const long o = ((long)plane * s.Ho + u) * s.Wo + v;
        stf(y, o, best);
        if (IS_MAX && am) am[o] = (uint8_t)bi;
    }
}

// dx rows p0 + r*d (r < R) of one column: they collect from dy rows p0 + (r-a)*d.
template <typename T, int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, PoolShape s)
{
    int plane, p0, q;
    pool_decode<R>(s, s.H, plane, p0, q);
    if (q >= s.W || p0 >= s.H) return;
    const T *dyp = dy + (long)plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + (long)plane * s.Ho * s.Wo : nullptr;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    // t indexes dy rows p0 + (t-(K-1))*d, t = 0 .. R+K-2; it feeds dx rows r = t-(K-1)+a
#pragma unroll
    for (int t = 0; t < R + K - 1; ++t) {
        const int u = p0 + (t - (K - 1)) * s.d;
        if (u < 0 || u >= s.Ho) continue;
#pragma unroll
        for (int b = 0; b < K; ++b) {
            const int v = q - b * s.d;
            if (v < 0 || v >= s.Wo) continue;
            const long o = (long)u * s.Wo + v;
            const float g = ldf(dyp, o);
            if (IS_MAX) {
                const int idx = amp[o];
#pragma unroll
                for (int a = 0; a < K; ++a) {
                    const int r = t - (K - 1) + a;
                    if (r >= 0 && r < R && idx == a * K + b) acc[r] += g;
                }
            } else {
#pragma unroll
                for (int a = 0; a < K; ++a) {
                    const int r = t - (K - 1) + a;
                    if (r >= 0 && r < R) acc[r] += g;
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = p0 + r * s.d;
        if (p >= s.H) break;
        const float v = IS_MAX ? acc[r] : acc[r] * (1.0f / (float)(K * K));
        stf(dx, ((long)plane * s.H + p) * s.W + q, v);
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
    constexpr int R = 8;
    PoolShape s = make_shape(N, C, H, W, k, d, R, H, W);
    const long tiled_blocks = (long)s.planes * s.row_groups * s.col_blocks;
    if (k == 2 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 2, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 3 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 3, R, IS_MAX><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
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
