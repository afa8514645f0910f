// Masked softmax cross-entropy at the last layer.  The pixel-of-interest mask of
// paper Sec. 4.3 keeps the prediction errors of chosen pixels and zeroes the
// rest; the chosen patches form one mini-batch whose gradients are averaged
// (Sec. 1.1).  Every pixel is visited and its error written whatever the mask
// holds, so the cost does not depend on the chosen subset.
//
// Four small launches, all reductions in a fixed order (no atomics):
//   1. per-block counts of mask != 0         -> ws.cnt[block]
//   2. one block sums them                   -> ws.total
//   3. per pixel: softmax, error map, loss   -> dscores, ws.loss[block]
//   4. one block sums the loss partials      -> loss[0] = -sum / total
#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;

// workspace: [0] total count (u32), [1..3] unused, then nblk u32 counts, then nblk float losses
static inline long n_blocks(long pixels) { return (pixels + kThreads - 1) / kThreads; }

size_t softmax_xent_ws_bytes(long pixels) { return (size_t)(4 + 2 * n_blocks(pixels)) * 4; }

__global__ void __launch_bounds__(kThreads)
mask_count_kernel(const uint8_t *__restrict__ mask, long pixels, uint32_t *__restrict__ cnt)
{
    __shared__ uint32_t sm[kThreads];
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    sm[threadIdx.x] = (idx < pixels && mask[idx] != 0) ? 1u : 0u;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) cnt[blockIdx.x] = sm[0];
}

__global__ void __launch_bounds__(kThreads)
count_total_kernel(const uint32_t *__restrict__ cnt, long nblk, uint32_t *__restrict__ total)
{
    __shared__ uint32_t sm[kThreads];
    uint32_t acc = 0;
    for (long i = threadIdx.x; i < nblk; i += kThreads) acc += cnt[i];
    sm[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) total[0] = sm[0];
}

template <typename TD>
__global__ void __launch_bounds__(kThreads)
softmax_xent_kernel(const float *__restrict__ scores, const int32_t *__restrict__ labels,
                    const uint8_t *__restrict__ mask, const uint32_t *__restrict__ total,
                    TD *__restrict__ dscores, float *__restrict__ loss_part, int Cls, long HW, long pixels)
{
    __shared__ float sm[kThreads];
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    float my_loss = 0.f;
    if (idx < pixels) {
        const long n = idx / HW, hw = idx % HW;
        const float *sp = scores + n * Cls * HW + hw;
        TD *dp = dscores + n * Cls * HW + hw;
        const uint32_t cnt = total[0];
        const bool chosen = mask[idx] != 0 && cnt > 0;
        if (!chosen) {
            for (int c = 0; c < Cls; ++c) stf(dp, (long)c * HW, 0.f);
        } else {
            const int lab = labels[idx];
            float mx = sp[0];
            for (int c = 1; c < Cls; ++c) mx = fmaxf(mx, sp[(long)c * HW]);
            float sum = 0.f;
            for (int c = 0; c < Cls; ++c) sum += expf(sp[(long)c * HW] - mx);
            const float inv = 1.0f / sum;
            const float invc = 1.0f / (float)cnt;
            for (int c = 0; c < Cls; ++c) {
                const float p = expf(sp[(long)c * HW] - mx) * inv;
                stf(dp, (long)c * HW, (p - (c == lab ? 1.f : 0.f)) * invc);
            }
            if (lab >= 0 && lab < Cls) my_loss = logf(sum) - (sp[(long)lab * HW] - mx);
        }
    }
    sm[threadIdx.x] = my_loss;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss_part[blockIdx.x] = sm[0];
}

__global__ void __launch_bounds__(kThreads)
loss_total_kernel(const float *__restrict__ part, long nblk, const uint32_t *__restrict__ total,
                  float *__restrict__ loss)
{
    __shared__ float sm[kThreads];
    float acc = 0.f;
    for (long i = threadIdx.x; i < nblk; i += kThreads) acc += part[i];
    sm[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = total[0] > 0 ? sm[0] / (float)total[0] : 0.f;
}

int launch_masked_softmax_xent(const float *scores, const int32_t *labels, const uint8_t *mask, float *loss,
                               void *dscores, dsk_dtype dt, int N, int Cls, int H, int W, void *ws,
                               hipStream_t st)
{
    const long HW = (long)H * W, pixels = (long)N * HW;
    const long nblk = n_blocks(pixels);
    uint32_t *total = (uint32_t *)ws;
    uint32_t *cnt = total + 4;
    float *lpart = (float *)(cnt + nblk);
    mask_count_kernel<<<dim3((unsigned)nblk), dim3(kThreads), 0, st>>>(mask, pixels, cnt);
    count_total_kernel<<<dim3(1), dim3(kThreads), 0, st>>>(cnt, nblk, total);
    if (dt == DSK_F32)
        softmax_xent_kernel<float><<<dim3((unsigned)nblk), dim3(kThreads), 0, st>>>(
            scores, labels, mask, total, (float *)dscores, lpart, Cls, HW, pixels);
    else
        softmax_xent_kernel<bf16><<<dim3((unsigned)nblk), dim3(kThreads), 0, st>>>(
            scores, labels, mask, total, (bf16 *)dscores, lpart, Cls, HW, pixels);
    loss_total_kernel<<<dim3(1), dim3(kThreads), 0, st>>>(lpart, nblk, total, loss);
    return check_launch();
}

} // namespace dsk
