// Image padding (paper Sec. 3.3) and the backward of the point-wise
// non-linearity layer.  Both are pure streaming kernels.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;

template <typename TO>
__global__ void __launch_bounds__(kThreads)
pad_image_kernel(const float *__restrict__ x, TO *__restrict__ xp, long planes, int H, int W, int lo, int Hp, int Wp)
{
    const long total = planes * Hp * Wp;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int q = (int)(idx % Wp);
    const int p = (int)((idx / Wp) % Hp);
    const long plane = idx / ((long)Wp * Hp);
    const int i = p - lo, j = q - lo;
    float v = 0.f;
    if (i >= 0 && i < H && j >= 0 && j < W) v = x[(plane * H + i) * W + j];
    stf(xp, idx, v);
}

template <typename T>
__global__ void __launch_bounds__(kThreads)
act_bwd_kernel(const T *__restrict__ y, T *__restrict__ dy, size_t count, int act)
{
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= count) return;
    const float yv = ldf(y, (long)idx);
    const float g = ldf(dy, (long)idx);
    const float f = (act == DSK_ACT_RELU) ? (yv > 0.f ? 1.f : 0.f) : (1.f - yv * yv);
    stf(dy, (long)idx, g * f);
}

// Fused backward of the non-linearity and bias gradient: one pass over the error map of a conv
// layer's output.  kBiasSplit workgroups per filter each take a contiguous share of every
// image's plane (coalesced), multiply in place and sum; a second tiny kernel adds the shares
// in a fixed order.
static constexpr int kBiasSplit = 32;

template <typename T>
__global__ void __launch_bounds__(kThreads)
act_bwd_bias_kernel(const T *__restrict__ y, T *__restrict__ dy, float *__restrict__ part, int N, int K, long plane,
                    int act)
{
    __shared__ float sm[kThreads];
    const int f = blockIdx.x / kBiasSplit, sp = blockIdx.x % kBiasSplit;
    const long share = (plane + kBiasSplit - 1) / kBiasSplit;
    const long lo = sp * share, hi = lo + share < plane ? lo + share : plane;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) {
        const long base = ((long)n * K + f) * plane;
        for (long t = lo + threadIdx.x; t < hi; t += kThreads) {
            float g = ldf(dy, base + t);
            if (act != DSK_ACT_NONE) {
                const float yv = ldf(y, base + t);
                g *= (act == DSK_ACT_RELU) ? (yv > 0.f ? 1.f : 0.f) : (1.f - yv * yv);
                stf(dy, base + t, g);
                g = ldf(dy, base + t);      // what the weight gradient will read (bf16: the rounded value)
            }
            acc += g;
        }
    }
    sm[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = sm[0];
}

__global__ void __launch_bounds__(kThreads)
bias_sum_kernel(const float *__restrict__ part, float *__restrict__ db, int K)
{
    const int f = blockIdx.x * kThreads + threadIdx.x;
    if (f >= K) return;
    float acc = 0.f;
    for (int sp = 0; sp < kBiasSplit; ++sp) acc += part[f * kBiasSplit + sp];
    db[f] = acc;
}

size_t act_bwd_bias_ws_bytes(int K) { return (size_t)K * kBiasSplit * sizeof(float); }

int launch_act_bwd_bias(const void *y, void *dy, float *db, int N, int K, long plane, int act, dsk_dtype t,
                        void *ws, hipStream_t st)
{
    float *part = (float *)ws;
    dim3 g((unsigned)(K * kBiasSplit)), th(kThreads);
    if (t == DSK_F32)
        act_bwd_bias_kernel<float><<<g, th, 0, st>>>((const float *)y, (float *)dy, part, N, K, plane, act);
    else
        act_bwd_bias_kernel<bf16><<<g, th, 0, st>>>((const bf16 *)y, (bf16 *)dy, part, N, K, plane, act);
    bias_sum_kernel<<<dim3((K + kThreads - 1) / kThreads), th, 0, st>>>(part, db, K);
    return check_launch();
}

int launch_pad_image(const float *x, void *xpad, int N, int C, int H, int W, int lo, int hi, dsk_dtype out,
                     hipStream_t st)
{
    const int Hp = H + lo + hi, Wp = W + lo + hi;
    const long planes = (long)N * C;
    const long total = planes * Hp * Wp;
    dim3 g((unsigned)((total + kThreads - 1) / kThreads)), t(kThreads);
    if (out == DSK_F32)
        pad_image_kernel<float><<<g, t, 0, st>>>(x, (float *)xpad, planes, H, W, lo, Hp, Wp);
    else
        pad_image_kernel<bf16><<<g, t, 0, st>>>(x, (bf16 *)xpad, planes, H, W, lo, Hp, Wp);
    return check_launch();
}

int launch_act_bwd(const void *y, void *dy, size_t count, int act, dsk_dtype t, hipStream_t st)
{
    if (act == DSK_ACT_NONE || count == 0) return DSK_OK;
    dim3 g((unsigned)((count + kThreads - 1) / kThreads)), th(kThreads);
    if (t == DSK_F32)
        act_bwd_kernel<float><<<g, th, 0, st>>>((const float *)y, (float *)dy, count, act);
    else
        act_bwd_kernel<bf16><<<g, th, 0, st>>>((const bf16 *)y, (bf16 *)dy, count, act);
    return check_launch();
}

} // namespace dsk
