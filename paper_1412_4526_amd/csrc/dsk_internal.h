// Internal declarations shared by libdsk's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dsk.h"

namespace dsk {

// bfloat16 storage type: the upper 16 bits of an IEEE fp32.
struct bf16 {
    uint16_t v;
};

__host__ __device__ inline float bf16_to_f32(bf16 h)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)h.v << 16;
    return c.f;
}

// round-to-nearest-even; NaN stays NaN (quiet)
__host__ __device__ inline bf16 f32_to_bf16(float f)
{
#ifdef __HIP_DEVICE_COMPILE__
    // the conversion instruction of the matrix-core generation: the same rounding, one instruction
    bf16 h;
    h.v = __builtin_bit_cast(uint16_t, (__bf16)f);
    return h;
#else
    union { uint32_t u; float f; } c;
    c.f = f;
    bf16 h;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) {
        h.v = (uint16_t)((c.u >> 16) | 0x0040u);
    } else {
        c.u += 0x7fffu + ((c.u >> 16) & 1u);
        h.v = (uint16_t)(c.u >> 16);
    }
    return h;
#endif
}

__device__ inline float ldf(const float *p, long i) { return p[i]; }
__device__ inline float ldf(const bf16 *p, long i) { return bf16_to_f32(p[i]); }
__device__ inline void stf(float *p, long i, float v) { p[i] = v; }
__device__ inline void stf(bf16 *p, long i, float v) { p[i] = f32_to_bf16(v); }

// Buffer loads: a 128-bit descriptor of [base, end) held in scalar registers, one per-lane
// offset and one scalar offset per load (both in elements), so that a load costs one scalar
// instruction besides itself.  Offsets at or beyond `end` read zero.
typedef __amdgpu_buffer_rsrc_t BufRsrc;
template <typename T>
__device__ inline BufRsrc buf_rsrc(const T *base, const T *end)
{
    const unsigned long bytes = (unsigned long)((const char *)end - (const char *)base);
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, bytes < 0xfffffffcul ? (int)(unsigned)bytes : (int)0xfffffffcu,
                                             0x00020000);
}
__device__ inline float buf_ld(BufRsrc r, const float *, unsigned lane_off, unsigned uniform_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)(lane_off * 4u), (int)(uniform_off * 4u), 0));
}
__device__ inline float buf_ld(BufRsrc r, const bf16 *, unsigned lane_off, unsigned uniform_off)
{
    bf16 v;
    v.v = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)(lane_off * 2u), (int)(uniform_off * 2u), 0);
    return bf16_to_f32(v);
}
__device__ inline int buf_ld(BufRsrc r, const uint8_t *, unsigned lane_off, unsigned uniform_off)
{
    return (int)(uint8_t)__builtin_amdgcn_raw_buffer_load_b8(r, (int)lane_off, (int)uniform_off, 0);
}
__device__ inline void buf_st(BufRsrc r, float *, unsigned lane_off, unsigned uniform_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)(lane_off * 4u), (int)(uniform_off * 4u), 0);
}
__device__ inline void buf_st(BufRsrc r, bf16 *, unsigned lane_off, unsigned uniform_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16(v).v, r, (int)(lane_off * 2u), (int)(uniform_off * 2u), 0);
}
__device__ inline void buf_st(BufRsrc r, uint8_t *, unsigned lane_off, unsigned uniform_off, int v)
{
    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)v, r, (int)lane_off, (int)uniform_off, 0);
}

// value a kernel computing in type T sees for an fp32 weight
template <typename T> __device__ inline float round_w(float w);
template <> __device__ inline float round_w<float>(float w) { return w; }
template <> __device__ inline float round_w<bf16>(float w) { return bf16_to_f32(f32_to_bf16(w)); }

__device__ inline float act_apply(int act, float z)
{
    if (act == DSK_ACT_RELU) return z > 0.f ? z : 0.f;
    if (act == DSK_ACT_TANH) return tanhf(z);
    return z;
}

struct ConvShape {
    int N, C, H, W, K, kh, kw, d, Ho, Wo;
    // Video (3-D) layers run as per-frame 2-D calls whose contraction also runs over the temporal taps: the
    // frames of a video [T][C][H][W] are a batch of images, and the planes of temporal tap e are those of the
    // frame e*dt further on.  All zero for a plain 2-D call.
    //  * gsize / gjump (forward: channels of x; backward-data: filters of dy): the contraction's planes come in
    //    groups of gsize; plane v of image slot b lies at (b*gsize + v)*plane + (v / gsize)*gjump elements.
    //  * bgroup / bskip (the tensor the call reads: x, or dy for backward-data; for the weight gradient: x):
    //    image n sits at slot n + n / bgroup * bskip (frames of the next video start bskip slots later).
    //  * in_extent: elements of that tensor, from its first, that may be read (0: N*C*H*W, or N*K*Ho*Wo).
    int gsize = 0;
    long gjump = 0;
    int bgroup = 0, bskip = 0;
    long in_extent = 0;
};

// where plane c of image n of the tensor a convolution call reads begins (Cin planes of hw elements per image)
__host__ __device__ inline long conv_in_offset(const ConvShape &s, int n, int c, int Cin, long hw)
{
    const long slot = s.bgroup ? n + (long)(n / s.bgroup) * s.bskip : n;
    if (!s.gsize) return (slot * Cin + c) * hw;
    return (slot * s.gsize + c) * hw + (long)(c / s.gsize) * s.gjump;
}

// ---- plain one-thread-per-output kernels (dsk_direct.hip) ----
int launch_conv_fwd_direct(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                           dsk_dtype in, dsk_dtype out, int act, hipStream_t st);
int launch_conv_bwd_data_direct(const void *dy, const float *w, void *dx, const ConvShape &s,
                                dsk_dtype in, dsk_dtype out, hipStream_t st);
int launch_conv_bwd_weight_direct(const void *x, const void *dy, float *dw, float *db, const ConvShape &s,
                                  dsk_dtype in, hipStream_t st);

// ---- matrix-core (MFMA) kernels (dsk_conv_mfma.hip) ----
size_t conv_ws_bytes(int which, const ConvShape &s, dsk_dtype in);
bool conv_mfma_supported(int which, const ConvShape &s, dsk_dtype in, dsk_dtype out);
int launch_conv_fwd_mfma(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                         dsk_dtype in, dsk_dtype out, int act, void *ws, hipStream_t st);
int launch_conv_bwd_data_mfma(const void *dy, const float *w, void *dx, const ConvShape &s,
                              dsk_dtype in, dsk_dtype out, void *ws, hipStream_t st);
int launch_conv_bwd_weight_mfma(const void *x, const void *dy, float *dw, float *db, const ConvShape &s,
                                dsk_dtype in, void *ws, hipStream_t st);
// backward-data of a 1 x 1 layer with the non-linearity backward and bias gradient of the layer below in its epilogue
bool conv_bwd_data_act_fused(const ConvShape &s, dsk_dtype in, dsk_dtype out);
size_t conv_bwd_data_act_ws_bytes(const ConvShape &s);
int launch_conv_bwd_data_act(const void *dy, const float *w, const void *x, void *dx, float *db, const ConvShape &s,
                             dsk_dtype t, int act, void *ws, hipStream_t st);

// kernel choice for one 2-D convolution call, as the entry points make it (dsk_api.hip)
int dispatch_conv_fwd(const void *x, const float *w, const float *b, void *y, const ConvShape &s, dsk_dtype in,
                      dsk_dtype out, int act, void *ws, hipStream_t st);
int dispatch_conv_bwd_data(const void *dy, const float *w, void *dx, const ConvShape &s, dsk_dtype in, dsk_dtype out,
                           void *ws, hipStream_t st);
int dispatch_conv_bwd_weight(const void *x, const void *dy, float *dw, float *db, const ConvShape &s, dsk_dtype in,
                             void *ws, hipStream_t st);

// ---- bf16 matrix-core kernels for forward / backward-data on bf16 maps (dsk_conv_bf16.hip) ----
size_t conv_bf16_ws_bytes(int which, const ConvShape &s);
bool conv_bf16_supported(int which, const ConvShape &s);
int launch_conv_fwd_bf16(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                         dsk_dtype out, int act, void *ws, hipStream_t st);
int launch_conv_bwd_data_bf16(const void *dy, const float *w, void *dx, const ConvShape &s, dsk_dtype out, void *ws,
                              hipStream_t st);

// ---- bf16 matrix-core kernel for the weight gradient on bf16 maps (dsk_bww_bf16.hip): square kernels of 3-5 taps
// a side; writes partial blocks part[S][kh*kw][Kp][Cp] for the reduce kernel of dsk_conv_mfma.hip
bool bww_bf16_shape(const ConvShape &s, int *Kp, int *Cp, int *S);
int launch_bww_bf16(const void *x, const void *dy, float *part, const ConvShape &s, hipStream_t st);

// ---- pooling, padding, activation, loss (dsk_pool.hip, dsk_misc.hip, dsk_loss.hip) ----
int launch_maxpool_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st);
int launch_maxpool_bwd(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st);
int launch_avgpool_fwd(const void *x, void *y, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st);
int launch_avgpool_bwd(const void *dy, void *dx, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st);
// 2 x 2 and 3 x 3 windows: a thread walks down a residue class of rows (dsk_pool_walk.hip)
bool pool_walk_ok(int N, int C, int H, int W, int k, int d, dsk_dtype t);
int launch_pool_walk_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d, bool is_max,
                         dsk_dtype t, hipStream_t st);
size_t pool_bwd_act_bias_ws_bytes(int N, int C, int H, int W, int k, int d, dsk_dtype t);
int launch_pool_walk_bwd(const void *dy, const uint8_t *am, void *dx, const void *yprev, float *db, int act, void *ws,
                         int N, int C, int H, int W, int k, int d, bool is_max, dsk_dtype t, hipStream_t st);
// fast scanning, the comparison method (dsk_fastscan.hip)
int launch_fs_pool(const void *in, void *out, bool is_max, int N, int D, int C, int hi, int wi, int k, int s, int ho, int wo,
                   dsk_dtype t, hipStream_t st);
int launch_fs_conv(const void *in, const float *w, const float *b, void *out, int N, int D, int C, int hi, int wi, int K, int k,
                   int s, int ho, int wo, int act, dsk_dtype t, hipStream_t st);
int launch_fs_assemble(const void *frag, void *out, int N, int D, int C, int hf, int wf, int H, int W, dsk_dtype ti, dsk_dtype to,
                       hipStream_t st);
int launch_pad_image(const float *x, void *xpad, int N, int C, int H, int W, int lo, int hi, dsk_dtype out,
                     hipStream_t st);
int launch_act_bwd(const void *y, void *dy, size_t count, int act, dsk_dtype t, hipStream_t st);
size_t act_bwd_bias_ws_bytes(int K);
int launch_act_bwd_bias(const void *y, void *dy, float *db, int N, int K, long plane, int act, dsk_dtype t,
                        void *ws, hipStream_t st);
size_t softmax_xent_ws_bytes(long pixels);
int launch_masked_softmax_xent(const float *scores, const int32_t *labels, const uint8_t *mask, float *loss,
                               void *dscores, dsk_dtype dt, int N, int Cls, int H, int W, void *ws,
                               hipStream_t st);

int static_scratch_of_current_device(void **out);

// Launch errors are sticky in the HIP runtime: an entry point forgets what the caller's earlier
// HIP calls may have left behind before its first launch, so that check_launch reports only its own.
inline void clear_errors()
{
    (void)hipGetLastError();
}
inline int check_launch()
{
    return hipGetLastError() == hipSuccess ? DSK_OK : DSK_ELAUNCH;
}

// multiprocessors of the current device (cached per device)
int device_cu_count();

} // namespace dsk
