// Fast scanning -- the method the paper compares itself with (Sec. 2; Sec. 3.6, last paragraph; Table 1) -- as an
// on-device comparator, forward only (the paper: "only supports forward propagation").
//
// Fast scanning keeps every layer's ORIGINAL stride s and runs a strided layer s*s times, once per starting
// offset (ay, ax), 0 <= ay, ax < s.  Each run yields one output "fragment"; after strided layers with strides
// s1, s2, ... there are (s1*s2*...)^2 fragments per image, and the fragments of the last layer are re-organised
// into the label map.  In whole-image terms fragment (fy, fx) at fragment spacing D holds the map's entries
// (fy + D*u, fx + D*v).  Stride-1 layers treat every fragment as a small dense image (here: the library's own
// convolution with d = 1 on the batch of fragments).
//
// Fragments are stored as a batch [N*D*D][C][h][w], index n*D*D + fy*D + fx, all with the size of the largest
// one, h = ceil(H/D); smaller fragments leave their last row / column unused (what is computed from it is never
// part of a valid entry downstream).
//
// The kernels are deliberately plain -- one thread per output entry, taps read at stride s with the run's
// offset -- because that access pattern IS the method: the paper's point is that it cannot use the memory
// system the way stride-1 sparse kernels can.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kFsThreads = 256;

struct FsShape {
    int N, D, C, hi, wi, K, k, s, ho, wo, act;
    long total;      // output entries
};

// out fragment (n, fy + D*ay, fx + D*ax) at spacing D*s, entry (u, v) <- taps (ay + s*u + a, ax + s*v + b) of in fragment (n, fy, fx)
__device__ inline void fs_decode(const FsShape &p, long idx, int &fo, int &c, int &u, int &v, int &fi, int &ay, int &ax)
{
    v = (int)(idx % p.wo); idx /= p.wo;
    u = (int)(idx % p.ho); idx /= p.ho;
    c = (int)(idx % p.K); idx /= p.K;
    fo = (int)idx;
    const int Do = p.D * p.s, per = Do * Do;
    const int n = fo / per, r = fo % per, fyo = r / Do, fxo = r % Do;
    ay = fyo / p.D; ax = fxo / p.D;
    fi = n * p.D * p.D + (fyo % p.D) * p.D + (fxo % p.D);
}

template <typename T, bool IS_MAX>
__global__ void __launch_bounds__(kFsThreads)
fs_pool_kernel(const T *__restrict__ in, T *__restrict__ out, FsShape p)
{
    const long idx = (long)blockIdx.x * kFsThreads + threadIdx.x;
    if (idx >= p.total) return;
    int fo, c, u, v, fi, ay, ax;
    fs_decode(p, idx, fo, c, u, v, fi, ay, ax);
    const T *src = in + ((long)fi * p.C + c) * p.hi * p.wi;
    float best = 0.f;
    bool any = false;
    for (int a = 0; a < p.k; ++a) {
        const int r = ay + p.s * u + a;
        if (r >= p.hi) break;
        for (int b = 0; b < p.k; ++b) {
            const int q = ax + p.s * v + b;
            if (q >= p.wi) break;
            const float t = ldf(src, (long)r * p.wi + q);
            if (IS_MAX) best = !any || t > best ? t : best;
            else best += t;
            any = true;
        }
    }
    if (!IS_MAX) best *= 1.0f / (float)(p.k * p.k);
    stf(out, idx, best);
}

template <typename T>
__global__ void __launch_bounds__(kFsThreads)
fs_conv_kernel(const T *__restrict__ in, const float *__restrict__ w, const float *__restrict__ bias, T *__restrict__ out, FsShape p)
{
    const long idx = (long)blockIdx.x * kFsThreads + threadIdx.x;
    if (idx >= p.total) return;
    int fo, f, u, v, fi, ay, ax;
    fs_decode(p, idx, fo, f, u, v, fi, ay, ax);
    float acc = bias ? bias[f] : 0.f;
    for (int c = 0; c < p.C; ++c) {
        const T *src = in + ((long)fi * p.C + c) * p.hi * p.wi;
        const float *wf = w + ((long)f * p.C + c) * p.k * p.k;
        for (int a = 0; a < p.k; ++a) {
            const int r = ay + p.s * u + a;
            if (r >= p.hi) break;
            for (int b = 0; b < p.k; ++b) {
                const int q = ax + p.s * v + b;
                if (q >= p.wi) break;
                acc += round_w<T>(wf[a * p.k + b]) * ldf(src, (long)r * p.wi + q);
            }
        }
    }
    stf(out, idx, act_apply(p.act, acc));
}

// label map out[n][c][i][j] = fragment (n, i % D, j % D), entry (i / D, j / D)
template <typename TI, typename TO>
__global__ void __launch_bounds__(kFsThreads)
fs_assemble_kernel(const TI *__restrict__ frag, TO *__restrict__ out, int N, int D, int C, int hf, int wf, int H, int W)
{
    const long total = (long)N * C * H * W;
    const long idx = (long)blockIdx.x * kFsThreads + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % W);
    const int i = (int)((idx / W) % H);
    const int c = (int)((idx / ((long)W * H)) % C);
    const int n = (int)(idx / ((long)W * H * C));
    const long f = (long)n * D * D + (long)(i % D) * D + (j % D);
    stf(out, idx, ldf(frag, ((f * C + c) * hf + i / D) * wf + j / D));
}

int launch_fs_pool(const void *in, void *out, bool is_max, int N, int D, int C, int hi, int wi, int k, int s, int ho, int wo,
                   dsk_dtype t, hipStream_t st)
{
    FsShape p{N, D, C, hi, wi, C, k, s, ho, wo, 0, (long)N * D * s * D * s * C * ho * wo};
    const dim3 grid((unsigned)((p.total + kFsThreads - 1) / kFsThreads)), block(kFsThreads);
    if (t == DSK_F32 && is_max) fs_pool_kernel<float, true><<<grid, block, 0, st>>>((const float *)in, (float *)out, p);
    else if (t == DSK_F32) fs_pool_kernel<float, false><<<grid, block, 0, st>>>((const float *)in, (float *)out, p);
    else if (is_max) fs_pool_kernel<bf16, true><<<grid, block, 0, st>>>((const bf16 *)in, (bf16 *)out, p);
    else fs_pool_kernel<bf16, false><<<grid, block, 0, st>>>((const bf16 *)in, (bf16 *)out, p);
    return check_launch();
}

int launch_fs_conv(const void *in, const float *w, const float *b, void *out, int N, int D, int C, int hi, int wi, int K, int k,
                   int s, int ho, int wo, int act, dsk_dtype t, hipStream_t st)
{
    FsShape p{N, D, C, hi, wi, K, k, s, ho, wo, act, (long)N * D * s * D * s * K * ho * wo};
    const dim3 grid((unsigned)((p.total + kFsThreads - 1) / kFsThreads)), block(kFsThreads);
    if (t == DSK_F32) fs_conv_kernel<float><<<grid, block, 0, st>>>((const float *)in, w, b, (float *)out, p);
    else fs_conv_kernel<bf16><<<grid, block, 0, st>>>((const bf16 *)in, w, b, (bf16 *)out, p);
    return check_launch();
}

int launch_fs_assemble(const void *frag, void *out, int N, int D, int C, int hf, int wf, int H, int W, dsk_dtype ti, dsk_dtype to,
                       hipStream_t st)
{
    const long total = (long)N * C * H * W;
    const dim3 grid((unsigned)((total + kFsThreads - 1) / kFsThreads)), block(kFsThreads);
    if (ti == DSK_F32 && to == DSK_F32) fs_assemble_kernel<float, float><<<grid, block, 0, st>>>((const float *)frag, (float *)out, N, D, C, hf, wf, H, W);
    else if (ti == DSK_F32) fs_assemble_kernel<float, bf16><<<grid, block, 0, st>>>((const float *)frag, (bf16 *)out, N, D, C, hf, wf, H, W);
    else if (to == DSK_F32) fs_assemble_kernel<bf16, float><<<grid, block, 0, st>>>((const bf16 *)frag, (float *)out, N, D, C, hf, wf, H, W);
    else fs_assemble_kernel<bf16, bf16><<<grid, block, 0, st>>>((const bf16 *)frag, (bf16 *)out, N, D, C, hf, wf, H, W);
    return check_launch();
}

} // namespace dsk
