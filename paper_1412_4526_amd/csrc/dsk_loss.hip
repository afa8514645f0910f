// Masked softmax cross-entropy at the last layer.  The pixel-of-interest mask of
// paper Sec. 4.3 keeps the prediction errors of chosen pixels and zeroes the
// rest; the chosen patches form one mini-batch whose gradients are averaged
// (Sec. 1.1).
//
// Two launches, every sum in a fixed order, no atomics and no fences:
//   1. mask_loss_kernel: up to kCountBlocks workgroups take a contiguous share of the
//      mask each, count its chosen pixels and add up their loss terms
//      -log p[label] (softmax with the class scores of a pixel held in registers);
//      wavefront shuffles, then LDS, reduce over the workgroup -> ws.cnt[b], ws.nll[b]
//   2. softmax_xent_kernel: every workgroup adds the counts (same order everywhere);
//      a thread owns one pixel, or four neighbouring ones where the planes allow
//      16-byte accesses, and writes their error entries; the first workgroup also
//      adds the loss terms                                        -> dscores, loss[0]
// An unchosen pixel gets zeros without its scores being read; the scores of a chosen
// pixel are read by both kernels.
#include <mutex>

#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;
static constexpr int kCountBlocks = 1024;      // at most; a share is a multiple of 1024 pixels

// workspace (32-bit words): [0..3] unused, [4 .. 4+kCountBlocks) counts, then kCountBlocks loss sums
static inline long n_blocks(long pixels) { return (pixels + kThreads - 1) / kThreads; }

size_t softmax_xent_ws_bytes(long) { return (size_t)(4 + 2 * kCountBlocks) * 4; }

// Scratch of dsk_masked_softmax_xent_static: the workspace (its size does not depend on the map), one copy per
// GPU, held until the process ends.
static constexpr size_t kStaticScratchBytes = (size_t)(4 + 2 * kCountBlocks) * 4;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

__device__ inline unsigned wave_sum(unsigned v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// sum over the workgroup, returned to every thread; sm: kThreads / 64 words
template <typename T>
__device__ inline T block_sum(T v, T *sm)
{
    v = wave_sum(v);
    __syncthreads();                      // sm may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    T t = sm[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) t += sm[w];
    return t;
}

// softmax of one pixel: e[c] = exp(s[c] - max), their sum, and s[label] - max.  CMAX: upper bound of the
// class count for which the scores stay in registers (one pass over them).
template <int CMAX>
__device__ inline void pixel_softmax(const float *sp, long HW, int Cls, int lab, float (&e)[CMAX], float &sum, float &zlab)
{
#pragma unroll
    for (int c = 0; c < CMAX; ++c) e[c] = c < Cls ? sp[(long)c * HW] : -INFINITY;
    float mx = e[0];
#pragma unroll
    for (int c = 1; c < CMAX; ++c) mx = fmaxf(mx, e[c]);
    sum = 0.f;
    zlab = 0.f;
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        zlab = c == lab ? e[c] - mx : zlab;
        e[c] = c < Cls ? expf(e[c] - mx) : 0.f;
        sum += e[c];
    }
}

// -log p[label] of one pixel (0 for a label outside [0, Cls))
template <int CMAX>
__device__ inline float pixel_nll(const float *sp, long HW, int Cls, int lab)
{
    if (lab < 0 || lab >= Cls) return 0.f;
    if constexpr (CMAX > 0) {
        float e[CMAX], sum, zlab;
        pixel_softmax<CMAX>(sp, HW, Cls, lab, e, sum, zlab);
        return logf(sum) - zlab;
    } else {
        float mx = sp[0];
        for (int c = 1; c < Cls; ++c) mx = fmaxf(mx, sp[(long)c * HW]);
        float sum = 0.f;
        for (int c = 0; c < Cls; ++c) sum += expf(sp[(long)c * HW] - mx);
        return logf(sum) - (sp[(long)lab * HW] - mx);
    }
}

template <int CMAX>
__global__ void __launch_bounds__(kThreads)
mask_loss_kernel(const float *__restrict__ scores, const int32_t *__restrict__ labels, const uint8_t *__restrict__ mask,
                 long pixels, long share, int Cls, long HW, uint32_t *__restrict__ ws)
{
    __shared__ unsigned smu[kThreads / 64];
    __shared__ float smf[kThreads / 64];
    const long lo = (long)blockIdx.x * share, hi = lo + share < pixels ? lo + share : pixels;
    unsigned cnt = 0;
    float nll = 0.f;
    auto pixel = [&](long q) {
        ++cnt;
        const long n = q / HW, hw = q - n * HW;
        nll += pixel_nll<CMAX>(scores + n * Cls * HW + hw, HW, Cls, labels[q]);
    };
    // 4 mask bytes per load (the mask is 16-byte aligned and a share is a multiple of 1024 pixels): neighbouring
    // threads take neighbouring pixels, so that the score loads of chosen pixels are coalesced where the mask is dense
    long t = lo + 4L * threadIdx.x;
    for (; t + 4 <= hi; t += 4L * kThreads) {
        const unsigned w = *(const unsigned *)(mask + t);
        if (w == 0u) continue;
        for (int i = 0; i < 4; ++i)
            if ((w >> (8 * i)) & 0xffu) pixel(t + i);
    }
    if (t < hi)
        for (long q = t; q < hi; ++q)
            if (mask[q] != 0) pixel(q);
    const unsigned total = block_sum(cnt, smu);
    const float loss = block_sum(nll, smf);
    if (threadIdx.x == 0) {
        ws[4 + blockIdx.x] = total;
        ((float *)ws)[4 + kCountBlocks + blockIdx.x] = loss;
    }
}

// V pixels per thread (4: the planes are multiples of four pixels, so four neighbouring error entries are one
// aligned 16-byte store)
template <typename TD, int CMAX, int V>
__global__ void __launch_bounds__(kThreads)
softmax_xent_kernel(const float *__restrict__ scores, const int32_t *__restrict__ labels,
                    const uint8_t *__restrict__ mask, const uint32_t *__restrict__ ws, int n_cnt,
                    TD *__restrict__ dscores, float *__restrict__ loss, int Cls, long HW, long pixels)
{
    __shared__ unsigned smu[kThreads / 64];
    __shared__ float smf[kThreads / 64];
    unsigned c_acc = 0;
    for (int i = threadIdx.x; i < n_cnt; i += kThreads) c_acc += ws[4 + i];
    const unsigned cnt = block_sum(c_acc, smu);
    if (blockIdx.x == 0) {
        float l_acc = 0.f;
        for (int i = threadIdx.x; i < n_cnt; i += kThreads) l_acc += ((const float *)ws)[4 + kCountBlocks + i];
        const float total = block_sum(l_acc, smf);
        if (threadIdx.x == 0) loss[0] = cnt > 0 ? total / (float)cnt : 0.f;
    }
    const long idx = ((long)blockIdx.x * kThreads + threadIdx.x) * V;
    if (idx >= pixels) return;
    const long n = idx / HW, hw = idx - n * HW;
    const float *sp = scores + n * Cls * HW + hw;
    TD *dp = dscores + n * Cls * HW + hw;
    const float invc = cnt > 0 ? 1.0f / (float)cnt : 0.f;
    unsigned mk;
    if constexpr (V == 4) mk = cnt > 0 ? *(const unsigned *)(mask + idx) : 0u;
    else mk = cnt > 0 && mask[idx] != 0;
    if (mk == 0u) {
        for (int c = 0; c < Cls; ++c) {
            if constexpr (V == 4 && sizeof(TD) == 4) *(float4 *)(dp + (long)c * HW) = make_float4(0.f, 0.f, 0.f, 0.f);
            else if constexpr (V == 4) *(uint2 *)(dp + (long)c * HW) = make_uint2(0u, 0u);
            else stf(dp, (long)c * HW, 0.f);
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const bool chosen = (mk >> (8 * j)) & 0xffu;
        if (!chosen) {
            for (int c = 0; c < Cls; ++c) stf(dp + j, (long)c * HW, 0.f);
            continue;
        }
        const int lab = labels[idx + j];
        if constexpr (CMAX > 0) {
            float e[CMAX], sum, zlab;
            pixel_softmax<CMAX>(sp + j, HW, Cls, lab, e, sum, zlab);
            const float inv = 1.0f / sum;
#pragma unroll
            for (int c = 0; c < CMAX; ++c)
                if (c < Cls) stf(dp + j, (long)c * HW, (e[c] * inv - (c == lab ? 1.f : 0.f)) * invc);
        } else {
            float mx = sp[j];
            for (int c = 1; c < Cls; ++c) mx = fmaxf(mx, sp[j + (long)c * HW]);
            float sum = 0.f;
            for (int c = 0; c < Cls; ++c) sum += expf(sp[j + (long)c * HW] - mx);
            const float inv = 1.0f / sum;
            for (int c = 0; c < Cls; ++c)
                stf(dp + j, (long)c * HW, (expf(sp[j + (long)c * HW] - mx) * inv - (c == lab ? 1.f : 0.f)) * invc);
        }
    }
}

template <typename TD, int CMAX>
static void launch_both(const float *scores, const int32_t *labels, const uint8_t *mask, uint32_t *ws, int n_cnt, long share,
                        TD *dscores, float *loss, int Cls, long HW, long pixels, hipStream_t st)
{
    mask_loss_kernel<CMAX><<<dim3((unsigned)n_cnt), dim3(kThreads), 0, st>>>(scores, labels, mask, pixels, share, Cls, HW, ws);
    if (HW % 4 == 0)
        softmax_xent_kernel<TD, CMAX, 4><<<dim3((unsigned)n_blocks((pixels + 3) / 4)), dim3(kThreads), 0, st>>>(
            scores, labels, mask, ws, n_cnt, dscores, loss, Cls, HW, pixels);
    else
        softmax_xent_kernel<TD, CMAX, 1><<<dim3((unsigned)n_blocks(pixels)), dim3(kThreads), 0, st>>>(
            scores, labels, mask, ws, n_cnt, dscores, loss, Cls, HW, pixels);
}

template <typename TD>
static void launch_softmax(const float *scores, const int32_t *labels, const uint8_t *mask, uint32_t *ws, int n_cnt, long share,
                           TD *dscores, float *loss, int Cls, long HW, long pixels, hipStream_t st)
{
#define DSK_SM(CM) launch_both<TD, CM>(scores, labels, mask, ws, n_cnt, share, dscores, loss, Cls, HW, pixels, st)
    if (Cls <= 4) DSK_SM(4);
    else if (Cls <= 16) DSK_SM(16);
    else if (Cls <= 40) DSK_SM(40);
    else if (Cls <= 64) DSK_SM(64);
    else DSK_SM(0);
#undef DSK_SM
}

int launch_masked_softmax_xent(const float *scores, const int32_t *labels, const uint8_t *mask, float *loss,
                               void *dscores, dsk_dtype dt, int N, int Cls, int H, int W, void *ws,
                               hipStream_t st)
{
    const long HW = (long)H * W, pixels = (long)N * HW;
    // shares of the mask: multiples of 1024 pixels (four per thread), at most kCountBlocks of them
    long share = (pixels + kCountBlocks - 1) / kCountBlocks;
    share = (share + 4 * kThreads - 1) / (4 * kThreads) * (4 * kThreads);
    const int n_cnt = (int)((pixels + share - 1) / share);
    if (dt == DSK_F32)
        launch_softmax<float>(scores, labels, mask, (uint32_t *)ws, n_cnt, share, (float *)dscores, loss, Cls, HW, pixels, st);
    else
        launch_softmax<bf16>(scores, labels, mask, (uint32_t *)ws, n_cnt, share, (bf16 *)dscores, loss, Cls, HW, pixels, st);
    return check_launch();
}

// The scratch array of the current device: the symbol is looked up once per device.
static constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

int static_scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DSK_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return DSK_ELAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DSK_OK;
}

} // namespace dsk
