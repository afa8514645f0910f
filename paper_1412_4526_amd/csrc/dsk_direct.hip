// Plain one-thread-per-output kernels for the three sparse-kernel convolution
// operators (paper Sec. 3.1-3.2 forward, Sec. 4.1 backward).  They handle every
// shape and dtype and serve as the on-device cross-check for the matrix-core
// kernels; consecutive threads touch consecutive addresses in every tap.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;

template <typename TI, typename TO>
__global__ void __launch_bounds__(kThreads)
conv_fwd_direct_kernel(const TI *__restrict__ x, const float *__restrict__ w, const float *__restrict__ b,
                       TO *__restrict__ y, ConvShape s, int act)
{
    const long total = (long)s.N * s.K * s.Ho * s.Wo;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int v = (int)(idx % s.Wo);
    const int u = (int)((idx / s.Wo) % s.Ho);
    const int f = (int)((idx / ((long)s.Wo * s.Ho)) % s.K);
    const int n = (int)(idx / ((long)s.Wo * s.Ho * s.K));
    float acc = b ? b[f] : 0.f;
    for (int c = 0; c < s.C; ++c) {
        const TI *xp = x + conv_in_offset(s, n, c, s.C, (long)s.H * s.W) + (long)u * s.W + v;
        const float *wp = w + ((long)f * s.C + c) * s.kh * s.kw;
        for (int a = 0; a < s.kh; ++a)
            for (int bb = 0; bb < s.kw; ++bb)
                acc = fmaf(round_w<TI>(wp[a * s.kw + bb]), ldf(xp, (long)a * s.d * s.W + bb * s.d), acc);
    }
    stf(y, idx, act_apply(act, acc));
}

template <typename TI, typename TO>
__global__ void __launch_bounds__(kThreads)
conv_bwd_data_direct_kernel(const TI *__restrict__ dy, const float *__restrict__ w, TO *__restrict__ dx,
                            ConvShape s)
{
    const long total = (long)s.N * s.C * s.H * s.W;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int q = (int)(idx % s.W);
    const int p = (int)((idx / s.W) % s.H);
    const int c = (int)((idx / ((long)s.W * s.H)) % s.C);
    const int n = (int)(idx / ((long)s.W * s.H * s.C));
    float acc = 0.f;
    for (int f = 0; f < s.K; ++f) {
        const TI *dyp = dy + conv_in_offset(s, n, f, s.K, (long)s.Ho * s.Wo);
        const float *wp = w + ((long)f * s.C + c) * s.kh * s.kw;
        for (int a = 0; a < s.kh; ++a) {
            const int u = p - a * s.d;
            if (u < 0 || u >= s.Ho) continue;
            for (int bb = 0; bb < s.kw; ++bb) {
                const int v = q - bb * s.d;
                if (v < 0 || v >= s.Wo) continue;
                acc = fmaf(round_w<TI>(wp[a * s.kw + bb]), ldf(dyp, (long)u * s.Wo + v), acc);
            }
        }
    }
    stf(dx, idx, acc);
}

// fixed-order tree reduction over the block; result valid in thread 0
__device__ inline float block_sum(float v, float *sm)
{
    sm[threadIdx.x] = v;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    return sm[0];
}

// one block per kernel entry (f, c, a, b); threads stride over the output pixels
template <typename TI>
__global__ void __launch_bounds__(kThreads)
conv_bwd_weight_direct_kernel(const TI *__restrict__ x, const TI *__restrict__ dy, float *__restrict__ dw,
                              ConvShape s)
{
    __shared__ float sm[kThreads];
    const int e = blockIdx.x;
    const int bb = e % s.kw;
    const int a = (e / s.kw) % s.kh;
    const int c = (e / (s.kw * s.kh)) % s.C;
    const int f = e / (s.kw * s.kh * s.C);
    const long plane = (long)s.Ho * s.Wo;
    float acc = 0.f;
    for (int n = 0; n < s.N; ++n) {
        const TI *dyp = dy + ((long)n * s.K + f) * plane;
        const TI *xp = x + conv_in_offset(s, n, c, s.C, (long)s.H * s.W) + (long)a * s.d * s.W + bb * s.d;
        for (long t = threadIdx.x; t < plane; t += kThreads) {
            const int u = (int)(t / s.Wo), v = (int)(t % s.Wo);
            acc = fmaf(ldf(dyp, t), ldf(xp, (long)u * s.W + v), acc);
        }
    }
    const float r = block_sum(acc, sm);
    if (threadIdx.x == 0) dw[e] = r;
}

template <typename TI>
__global__ void __launch_bounds__(kThreads)
conv_bwd_bias_direct_kernel(const TI *__restrict__ dy, float *__restrict__ db, ConvShape s)
{
    __shared__ float sm[kThreads];
    const int f = blockIdx.x;
    const long plane = (long)s.Ho * s.Wo;
    float acc = 0.f;
    for (int n = 0; n < s.N; ++n) {
        const TI *dyp = dy + ((long)n * s.K + f) * plane;
        for (long t = threadIdx.x; t < plane; t += kThreads) acc += ldf(dyp, t);
    }
    const float r = block_sum(acc, sm);
    if (threadIdx.x == 0) db[f] = r;
}

static inline unsigned blocks_for(long total) { return (unsigned)((total + kThreads - 1) / kThreads); }

int launch_conv_fwd_direct(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                           dsk_dtype in, dsk_dtype out, int act, hipStream_t st)
{
    const long total = (long)s.N * s.K * s.Ho * s.Wo;
    dim3 g(blocks_for(total)), t(kThreads);
    if (in == DSK_F32 && out == DSK_F32)
        conv_fwd_direct_kernel<float, float><<<g, t, 0, st>>>((const float *)x, w, b, (float *)y, s, act);
    else if (in == DSK_BF16 && out == DSK_BF16)
        conv_fwd_direct_kernel<bf16, bf16><<<g, t, 0, st>>>((const bf16 *)x, w, b, (bf16 *)y, s, act);
    else if (in == DSK_BF16 && out == DSK_F32)
        conv_fwd_direct_kernel<bf16, float><<<g, t, 0, st>>>((const bf16 *)x, w, b, (float *)y, s, act);
    else
        conv_fwd_direct_kernel<float, bf16><<<g, t, 0, st>>>((const float *)x, w, b, (bf16 *)y, s, act);
    return check_launch();
}

int launch_conv_bwd_data_direct(const void *dy, const float *w, void *dx, const ConvShape &s,
                                dsk_dtype in, dsk_dtype out, hipStream_t st)
{
    const long total = (long)s.N * s.C * s.H * s.W;
    dim3 g(blocks_for(total)), t(kThreads);
    if (in == DSK_F32 && out == DSK_F32)
        conv_bwd_data_direct_kernel<float, float><<<g, t, 0, st>>>((const float *)dy, w, (float *)dx, s);
    else if (in == DSK_BF16 && out == DSK_BF16)
        conv_bwd_data_direct_kernel<bf16, bf16><<<g, t, 0, st>>>((const bf16 *)dy, w, (bf16 *)dx, s);
    else if (in == DSK_BF16 && out == DSK_F32)
        conv_bwd_data_direct_kernel<bf16, float><<<g, t, 0, st>>>((const bf16 *)dy, w, (float *)dx, s);
    else
        conv_bwd_data_direct_kernel<float, bf16><<<g, t, 0, st>>>((const float *)dy, w, (bf16 *)dx, s);
    return check_launch();
}

int launch_conv_bwd_weight_direct(const void *x, const void *dy, float *dw, float *db, const ConvShape &s,
                                  dsk_dtype in, hipStream_t st)
{
    dim3 g((unsigned)((long)s.K * s.C * s.kh * s.kw)), t(kThreads);
    if (in == DSK_F32)
        conv_bwd_weight_direct_kernel<float><<<g, t, 0, st>>>((const float *)x, (const float *)dy, dw, s);
    else
        conv_bwd_weight_direct_kernel<bf16><<<g, t, 0, st>>>((const bf16 *)x, (const bf16 *)dy, dw, s);
    int rc = check_launch();
    if (rc != DSK_OK || !db) return rc;
    if (in == DSK_F32)
        conv_bwd_bias_direct_kernel<float><<<dim3(s.K), t, 0, st>>>((const float *)dy, db, s);
    else
        conv_bwd_bias_direct_kernel<bf16><<<dim3(s.K), t, 0, st>>>((const bf16 *)dy, db, s);
    return check_launch();
}

} // namespace dsk
