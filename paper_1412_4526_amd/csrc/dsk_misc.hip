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

typedef float misc_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned misc_u32x2 __attribute__((ext_vector_type(2)));

// four consecutive elements with one 16-byte (fp32) or 8-byte (bf16) access; i is a multiple of 4
// elements from a base that is aligned likewise
__device__ inline void ld4(const float *p, long i, float (&v)[4])
{
    const misc_f32x4 t = *(const misc_f32x4 *)(p + i);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
__device__ inline void ld4(const bf16 *p, long i, float (&v)[4])
{
    const misc_u32x2 t = *(const misc_u32x2 *)(p + i);
    const unsigned a = t[0], b = t[1];
    v[0] = __builtin_bit_cast(float, a << 16); v[1] = __builtin_bit_cast(float, a & 0xffff0000u);
    v[2] = __builtin_bit_cast(float, b << 16); v[3] = __builtin_bit_cast(float, b & 0xffff0000u);
}
// returns in v what was stored (bf16: the rounded values)
__device__ inline void st4(float *p, long i, float (&v)[4])
{
    const misc_f32x4 t = {v[0], v[1], v[2], v[3]};
    *(misc_f32x4 *)(p + i) = t;
}
__device__ inline void st4(bf16 *p, long i, float (&v)[4])
{
    unsigned h[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        h[j] = f32_to_bf16(v[j]).v;
        v[j] = __builtin_bit_cast(float, h[j] << 16);
    }
    const misc_u32x2 t = {h[0] | h[1] << 16, h[2] | h[3] << 16};
    *(misc_u32x2 *)(p + i) = t;
}

// VEC: the maps are 16-byte (bf16: 8-byte) aligned, so a thread moves four elements per memory
// instruction (the vector memory path takes as long for a 4-byte access per lane as for a
// 16-byte one).
template <typename T, bool VEC>
__global__ void __launch_bounds__(kThreads)
act_bwd_bias_kernel(const T *__restrict__ y, T *__restrict__ dy, float *__restrict__ part, int N, int K, long plane,
                    long share, int act)
{
    __shared__ float sm[kThreads];
    const int f = blockIdx.x / kBiasSplit, sp = blockIdx.x % kBiasSplit;
    const long lo = sp * share, hi = lo + share < plane ? lo + share : plane;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) {
        const long base = ((long)n * K + f) * plane;
        if (VEC) {
            // elements before the first and after the last aligned group of four: one thread each
            const long head = (4 - ((base + lo) & 3)) & 3;
            const long vb = lo + head < hi ? lo + head : hi, ve = vb + (hi - vb) / 4 * 4;
            float a4[4] = {0.f, 0.f, 0.f, 0.f};
            for (long t = vb + 4 * threadIdx.x; t < ve; t += 4 * kThreads) {
                float g[4];
                ld4(dy, base + t, g);
                if (act != DSK_ACT_NONE) {
                    float yv[4];
                    ld4(y, base + t, yv);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        g[j] *= (act == DSK_ACT_RELU) ? (yv[j] > 0.f ? 1.f : 0.f) : (1.f - yv[j] * yv[j]);
                    st4(dy, base + t, g);      // g: what the weight gradient will read (bf16: the rounded value)
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) a4[j] += g[j];
            }
            acc += (a4[0] + a4[1]) + (a4[2] + a4[3]);
            const long n_edge = (vb - lo) + (hi - ve);      // at most 6
            if ((long)threadIdx.x < n_edge) {
                const long t = (long)threadIdx.x < vb - lo ? lo + threadIdx.x : ve + (threadIdx.x - (vb - lo));
                float g = ldf(dy, base + t);
                if (act != DSK_ACT_NONE) {
                    const float yv = ldf(y, base + t);
                    g *= (act == DSK_ACT_RELU) ? (yv > 0.f ? 1.f : 0.f) : (1.f - yv * yv);
                    stf(dy, base + t, g);
                    g = ldf(dy, base + t);
                }
                acc += g;
            }
            continue;
        }
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
    const long share = (plane + kBiasSplit - 1) / kBiasSplit;
    const size_t esz = t == DSK_F32 ? 4 : 2;
    const bool vec = (uintptr_t)y % (4 * esz) == 0 && (uintptr_t)dy % (4 * esz) == 0;
    if (t == DSK_F32 && vec)
        act_bwd_bias_kernel<float, true><<<g, th, 0, st>>>((const float *)y, (float *)dy, part, N, K, plane, share, act);
    else if (t == DSK_F32)
        act_bwd_bias_kernel<float, false><<<g, th, 0, st>>>((const float *)y, (float *)dy, part, N, K, plane, share, act);
    else if (vec)
        act_bwd_bias_kernel<bf16, true><<<g, th, 0, st>>>((const bf16 *)y, (bf16 *)dy, part, N, K, plane, share, act);
    else
        act_bwd_bias_kernel<bf16, false><<<g, th, 0, st>>>((const bf16 *)y, (bf16 *)dy, part, N, K, plane, share, act);
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
