// C-ABI entry points of libdsk: argument validation (before any launch),
// Algorithm 1's host-side planner, and dispatch to the kernels.
#include <mutex>

#include "dsk_internal.h"

using namespace dsk;

namespace {

// kernel selection of the calling thread (a diagnostic switch; nothing is shared between threads)
thread_local int g_conv_algo = 0;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad_ptr(const void *p) { return p == nullptr || !aligned16(p); }
inline bool bad_dtype(int t) { return t != DSK_F32 && t != DSK_BF16; }
constexpr long kMaxElems = 0x7fffffffL;

// Validates a conv problem and fills the derived shape.
int conv_shape(int N, int C, int H, int W, int K, int kh, int kw, int d, ConvShape *s)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || kh < 1 || kw < 1 || d < 1) return DSK_EINVAL;
    const long Ho = (long)H - (long)(kh - 1) * d, Wo = (long)W - (long)(kw - 1) * d;
    if (Ho < 1 || Wo < 1) return DSK_ESHAPE;
    if ((long)N * C * H * W > kMaxElems || (long)N * K * Ho * Wo > kMaxElems ||
        (long)K * C * kh * kw > kMaxElems)
        return DSK_ESHAPE;
    *s = ConvShape{N, C, H, W, K, kh, kw, d, (int)Ho, (int)Wo};
    return DSK_OK;
}

int pool_check(const void *a, const void *b, int N, int C, int H, int W, int k, int d, int t)
{
    if (bad_ptr(a) || bad_ptr(b)) return DSK_EINVAL;
    if (N < 1 || C < 1 || H < 1 || W < 1 || k < 1 || d < 1) return DSK_EINVAL;
    if (bad_dtype(t)) return DSK_EINVAL;
    if (k * (long)k > 255) return DSK_ESHAPE;
    const long Ho = (long)H - (long)(k - 1) * d, Wo = (long)W - (long)(k - 1) * d;
    if (Ho < 1 || Wo < 1) return DSK_ESHAPE;
    if ((long)N * C * H * W > kMaxElems) return DSK_ESHAPE;
    if ((long)H * W >= (1L << 30)) return DSK_ESHAPE;      // 32-bit byte offsets inside a plane
    return DSK_OK;
}

} // namespace

namespace dsk {
// Kernel choice for one 2-D convolution call (also the per-frame calls of the video layers): the bf16 matrix
// cores for plain calls on bf16 maps they take, else the fp32 matrix cores, else the plain kernels.
static bool plain2d(const ConvShape &s) { return s.gsize == 0 && s.bgroup == 0; }

int dispatch_conv_fwd(const void *x, const float *w, const float *b, void *y, const ConvShape &s, dsk_dtype in,
                      dsk_dtype out, int act, void *ws, hipStream_t st)
{
    if (g_conv_algo == 0 && in == DSK_BF16 && plain2d(s) && conv_bf16_supported(DSK_WS_CONV_FWD, s))
        return launch_conv_fwd_bf16(x, w, b, y, s, out, act, ws, st);
    if (g_conv_algo != 1 && conv_mfma_supported(DSK_WS_CONV_FWD, s, in, out))
        return launch_conv_fwd_mfma(x, w, b, y, s, in, out, act, ws, st);
    return launch_conv_fwd_direct(x, w, b, y, s, in, out, act, st);
}

int dispatch_conv_bwd_data(const void *dy, const float *w, void *dx, const ConvShape &s, dsk_dtype in, dsk_dtype out,
                           void *ws, hipStream_t st)
{
    if (g_conv_algo == 0 && in == DSK_BF16 && plain2d(s) && conv_bf16_supported(DSK_WS_CONV_BWD_DATA, s))
        return launch_conv_bwd_data_bf16(dy, w, dx, s, out, ws, st);
    if (g_conv_algo != 1 && conv_mfma_supported(DSK_WS_CONV_BWD_DATA, s, in, out))
        return launch_conv_bwd_data_mfma(dy, w, dx, s, in, out, ws, st);
    return launch_conv_bwd_data_direct(dy, w, dx, s, in, out, st);
}

int dispatch_conv_bwd_weight(const void *x, const void *dy, float *dw, float *db, const ConvShape &s, dsk_dtype in,
                             void *ws, hipStream_t st)
{
    if (g_conv_algo != 1 && conv_mfma_supported(DSK_WS_CONV_BWD_WEIGHT, s, in, DSK_F32))
        return launch_conv_bwd_weight_mfma(x, dy, dw, db, s, in, ws, st);
    return launch_conv_bwd_weight_direct(x, dy, dw, db, s, in, st);
}

int device_cu_count()
{
    static std::mutex mu;
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}
} // namespace dsk

extern "C" {

const char *dsk_status_string(int status)
{
    switch (status) {
    case DSK_OK: return "DSK_OK";
    case DSK_EINVAL: return "DSK_EINVAL: null or misaligned pointer, non-positive size or spacing, or bad enum";
    case DSK_ESHAPE: return "DSK_ESHAPE: empty output, kernel too large, or tensor too large";
    case DSK_EDTYPE: return "DSK_EDTYPE: unsupported dtype combination";
    case DSK_EWORKSPACE: return "DSK_EWORKSPACE: workspace missing or too small";
    case DSK_ELAUNCH: return "DSK_ELAUNCH: HIP launch error";
    default: return "unknown dsk status";
    }
}

// ---- fast scanning (comparison method) ----
static int fs_check(int N, int D, int C, int hi, int wi, int K, int k, int s, int ho, int wo)
{
    if (N < 1 || D < 1 || C < 1 || hi < 1 || wi < 1 || K < 1 || k < 1 || s < 1 || ho < 1 || wo < 1) return DSK_EINVAL;
    if ((long)D * s > 4096) return DSK_ESHAPE;
    const long fi = (long)N * D * D, fo = fi * s * s;
    if (fi * C * hi * wi > kMaxElems || fo * K * ho * wo > kMaxElems) return DSK_ESHAPE;
    // the last entry of the run with offset 0 has its first tap inside the fragment
    if ((long)s * (ho - 1) >= hi || (long)s * (wo - 1) >= wi) return DSK_ESHAPE;
    return DSK_OK;
}

int dsk_fs_pool_fwd(int kind, const void *in, void *out, int N, int D, int C, int hi, int wi, int k, int s, int ho, int wo,
                    dsk_dtype t, void *stream)
{
    if (kind != DSK_MAXPOOL && kind != DSK_AVGPOOL) return DSK_EINVAL;
    if (bad_ptr(in) || bad_ptr(out) || bad_dtype(t)) return DSK_EINVAL;
    const int rc = fs_check(N, D, C, hi, wi, C, k, s, ho, wo);
    if (rc != DSK_OK) return rc;
    clear_errors();
    return launch_fs_pool(in, out, kind == DSK_MAXPOOL, N, D, C, hi, wi, k, s, ho, wo, t, (hipStream_t)stream);
}

int dsk_fs_conv_fwd(const void *in, const float *w, const float *b, void *out, int N, int D, int C, int hi, int wi, int K,
                    int k, int s, int ho, int wo, dsk_act act, dsk_dtype t, void *stream)
{
    if (bad_ptr(in) || bad_ptr(w) || bad_ptr(out) || (b && !aligned16(b)) || bad_dtype(t)) return DSK_EINVAL;
    if (act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    const int rc = fs_check(N, D, C, hi, wi, K, k, s, ho, wo);
    if (rc != DSK_OK) return rc;
    clear_errors();
    return launch_fs_conv(in, w, b, out, N, D, C, hi, wi, K, k, s, ho, wo, act, t, (hipStream_t)stream);
}

int dsk_fs_assemble(const void *frag, void *out, int N, int D, int C, int hf, int wf, int H, int W, dsk_dtype tin,
                    dsk_dtype tout, void *stream)
{
    if (bad_ptr(frag) || bad_ptr(out) || bad_dtype(tin) || bad_dtype(tout)) return DSK_EINVAL;
    if (N < 1 || D < 1 || C < 1 || hf < 1 || wf < 1 || H < 1 || W < 1) return DSK_EINVAL;
    if ((long)(H - 1) / D >= hf || (long)(W - 1) / D >= wf) return DSK_ESHAPE;      // the fragments do not cover the map
    if ((long)N * D * D * C * hf * wf > kMaxElems || (long)N * C * H * W > kMaxElems) return DSK_ESHAPE;
    clear_errors();
    return launch_fs_assemble(frag, out, N, D, C, hf, wf, H, W, tin, tout, (hipStream_t)stream);
}

int dsk_set_conv_algo(int algo)
{
    const int prev = g_conv_algo;
    if (algo >= 0 && algo <= 2) g_conv_algo = algo;
    return prev;
}

int dsk_plan(const dsk_layer *layers, int L, int C0, int H, int W, int n,
             dsk_layer_plan *out, int *rf, int *pad_lo, int *pad_hi)
{
    if (!layers || !out || L < 1 || C0 < 1 || H < 1 || W < 1 || n < 0) return DSK_EINVAL;
    // pass 1: spacings and receptive field (Algorithm 1: d starts at 1, d <- d * d_k after layer k)
    long d = 1, field = 1;
    for (int l = 0; l < L; ++l) {
        const dsk_layer &ly = layers[l];
        if (ly.kind != DSK_CONV && ly.kind != DSK_MAXPOOL && ly.kind != DSK_AVGPOOL) return DSK_EINVAL;
        if (ly.k < 1 || ly.s < 1) return DSK_EINVAL;
        if (ly.kind == DSK_CONV && (ly.K < 1 || ly.act < DSK_ACT_NONE || ly.act > DSK_ACT_TANH)) return DSK_EINVAL;
        if (ly.kind != DSK_CONV && (long)ly.k * ly.k > 255) return DSK_ESHAPE;
        field += (long)(ly.k - 1) * d;
        d *= ly.s;
        if (d > (1 << 20) || field > (1 << 24)) return DSK_ESHAPE;
    }
    const long patch = n == 0 ? field : n;
    if (patch < field) return DSK_ESHAPE;
    const long lo = patch / 2, hi = field - 1 - lo;
    if (hi < 0) return DSK_ESHAPE;
    // pass 2: shapes on the padded image
    long h = (long)H + field - 1, w = (long)W + field - 1;
    int c = C0;
    d = 1;
    for (int l = 0; l < L; ++l) {
        const dsk_layer &ly = layers[l];
        dsk_layer_plan &p = out[l];
        p.kind = ly.kind;
        p.act = ly.kind == DSK_CONV ? ly.act : DSK_ACT_NONE;
        p.C = c;
        p.K = ly.kind == DSK_CONV ? ly.K : c;
        p.k = ly.k;
        p.d = (int)d;
        p.H = (int)h;
        p.W = (int)w;
        h -= (long)(ly.k - 1) * d;
        w -= (long)(ly.k - 1) * d;
        p.Ho = (int)h;
        p.Wo = (int)w;
        c = p.K;
        d *= ly.s;
    }
    if (rf) *rf = (int)field;
    if (pad_lo) *pad_lo = (int)lo;
    if (pad_hi) *pad_hi = (int)hi;
    return DSK_OK;
}

int dsk_pad_image(const float *x, void *xpad, int N, int C, int H, int W, int lo, int hi, dsk_dtype out,
                  void *stream)
{
    if (bad_ptr(x) || bad_ptr(xpad)) return DSK_EINVAL;
    if (N < 1 || C < 1 || H < 1 || W < 1 || lo < 0 || hi < 0 || bad_dtype(out)) return DSK_EINVAL;
    if ((long)N * C * ((long)H + lo + hi) * ((long)W + lo + hi) > kMaxElems) return DSK_ESHAPE;
    clear_errors();
    return launch_pad_image(x, xpad, N, C, H, W, lo, hi, out, (hipStream_t)stream);
}

size_t dsk_conv_workspace_bytes(int which, int N, int C, int H, int W, int K, int kh, int kw, int d,
                                dsk_dtype in)
{
    ConvShape s;
    if (conv_shape(N, C, H, W, K, kh, kw, d, &s) != DSK_OK || bad_dtype(in)) return 0;
    return conv_ws_bytes(which, s, in);
}

int dsk_conv_fwd(const void *x, const float *w, const float *b, void *y,
                 int N, int C, int H, int W, int K, int kh, int kw, int d,
                 dsk_dtype in, dsk_dtype out, dsk_act act, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_ptr(x) || bad_ptr(w) || bad_ptr(y) || (b && !aligned16(b))) return DSK_EINVAL;
    if (bad_dtype(in) || bad_dtype(out) || act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    ConvShape s;
    int rc = conv_shape(N, C, H, W, K, kh, kw, d, &s);
    if (rc != DSK_OK) return rc;
    const size_t need = conv_ws_bytes(DSK_WS_CONV_FWD, s, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    clear_errors();
    return dispatch_conv_fwd(x, w, b, y, s, in, out, act, ws, (hipStream_t)stream);
}

int dsk_conv_bwd_data(const void *dy, const float *w, void *dx,
                      int N, int C, int H, int W, int K, int kh, int kw, int d,
                      dsk_dtype in, dsk_dtype out, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_ptr(dy) || bad_ptr(w) || bad_ptr(dx)) return DSK_EINVAL;
    if (bad_dtype(in) || bad_dtype(out)) return DSK_EINVAL;
    ConvShape s;
    int rc = conv_shape(N, C, H, W, K, kh, kw, d, &s);
    if (rc != DSK_OK) return rc;
    const size_t need = conv_ws_bytes(DSK_WS_CONV_BWD_DATA, s, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    clear_errors();
    return dispatch_conv_bwd_data(dy, w, dx, s, in, out, ws, (hipStream_t)stream);
}

size_t dsk_conv_bwd_data_act_bias_workspace_bytes(int N, int C, int H, int W, int K, int kh, int kw, int d,
                                                  dsk_dtype in, dsk_dtype out)
{
    ConvShape s;
    if (conv_shape(N, C, H, W, K, kh, kw, d, &s) != DSK_OK || bad_dtype(in) || bad_dtype(out)) return 0;
    size_t need = conv_ws_bytes(DSK_WS_CONV_BWD_DATA, s, in);
    const size_t a = act_bwd_bias_ws_bytes(C);
    if (a > need) need = a;
    if (conv_bwd_data_act_fused(s, in, out)) {
        const size_t f = conv_bwd_data_act_ws_bytes(s);
        if (f > need) need = f;
    }
    return need;
}

int dsk_conv_bwd_data_act_bias(const void *dy, const float *w, const void *x, void *dx, float *db,
                               int N, int C, int H, int W, int K, int kh, int kw, int d,
                               dsk_dtype in, dsk_dtype out, dsk_act act, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_ptr(dy) || bad_ptr(w) || bad_ptr(dx) || bad_ptr(db)) return DSK_EINVAL;
    if (bad_dtype(in) || bad_dtype(out) || act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    if (act != DSK_ACT_NONE && bad_ptr(x)) return DSK_EINVAL;
    ConvShape s;
    int rc = conv_shape(N, C, H, W, K, kh, kw, d, &s);
    if (rc != DSK_OK) return rc;
    const size_t need = dsk_conv_bwd_data_act_bias_workspace_bytes(N, C, H, W, K, kh, kw, d, in, out);
    if (ws == nullptr || !aligned16(ws) || ws_bytes < need) return DSK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    clear_errors();
    if (g_conv_algo != 1 && conv_bwd_data_act_fused(s, in, out))
        return launch_conv_bwd_data_act(dy, w, x, dx, db, s, out, act, ws, st);
    // other shapes: the two passes one after the other
    rc = dispatch_conv_bwd_data(dy, w, dx, s, in, out, ws, st);
    if (rc != DSK_OK) return rc;
    return launch_act_bwd_bias(x, dx, db, N, C, (long)H * W, act, out, ws, st);
}

int dsk_conv_bwd_weight(const void *x, const void *dy, float *dw, float *db,
                        int N, int C, int H, int W, int K, int kh, int kw, int d,
                        dsk_dtype in, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_ptr(x) || bad_ptr(dy) || bad_ptr(dw) || (db && !aligned16(db))) return DSK_EINVAL;
    if (bad_dtype(in)) return DSK_EINVAL;
    ConvShape s;
    int rc = conv_shape(N, C, H, W, K, kh, kw, d, &s);
    if (rc != DSK_OK) return rc;
    const size_t need = conv_ws_bytes(DSK_WS_CONV_BWD_WEIGHT, s, in);
    if (need > 0 && (ws == nullptr || !aligned16(ws) || ws_bytes < need)) return DSK_EWORKSPACE;
    clear_errors();
    return dispatch_conv_bwd_weight(x, dy, dw, db, s, in, ws, (hipStream_t)stream);
}

int dsk_maxpool_fwd(const void *x, void *y, uint8_t *argmax, int N, int C, int H, int W, int k, int d,
                    dsk_dtype t, void *stream)
{
    int rc = pool_check(x, y, N, C, H, W, k, d, t);
    if (rc != DSK_OK) return rc;
    if (argmax && !aligned16(argmax)) return DSK_EINVAL;
    clear_errors();
    return launch_maxpool_fwd(x, y, argmax, N, C, H, W, k, d, t, (hipStream_t)stream);
}

int dsk_maxpool_bwd(const void *dy, const uint8_t *argmax, void *dx, int N, int C, int H, int W, int k, int d,
                    dsk_dtype t, void *stream)
{
    int rc = pool_check(dy, dx, N, C, H, W, k, d, t);
    if (rc != DSK_OK) return rc;
    if (bad_ptr(argmax)) return DSK_EINVAL;
    clear_errors();
    return launch_maxpool_bwd(dy, argmax, dx, N, C, H, W, k, d, t, (hipStream_t)stream);
}

int dsk_avgpool_fwd(const void *x, void *y, int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream)
{
    int rc = pool_check(x, y, N, C, H, W, k, d, t);
    if (rc != DSK_OK) return rc;
    clear_errors();
    return launch_avgpool_fwd(x, y, N, C, H, W, k, d, t, (hipStream_t)stream);
}

int dsk_avgpool_bwd(const void *dy, void *dx, int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream)
{
    int rc = pool_check(dy, dx, N, C, H, W, k, d, t);
    if (rc != DSK_OK) return rc;
    clear_errors();
    return launch_avgpool_bwd(dy, dx, N, C, H, W, k, d, t, (hipStream_t)stream);
}

size_t dsk_pool_bwd_act_bias_workspace_bytes(int kind, int N, int C, int H, int W, int k, int d, dsk_dtype t)
{
    if ((kind != DSK_MAXPOOL && kind != DSK_AVGPOOL) || bad_dtype(t)) return 0;
    if (N < 1 || C < 1 || H < 1 || W < 1 || k < 1 || d < 1 || (long)H - (long)(k - 1) * d < 1 || (long)W - (long)(k - 1) * d < 1)
        return 0;
    const size_t a = act_bwd_bias_ws_bytes(C);
    const size_t b = pool_walk_ok(N, C, H, W, k, d, t) ? pool_bwd_act_bias_ws_bytes(N, C, H, W, k, d, t) : 0;
    return a > b ? a : b;
}

int dsk_pool_bwd_act_bias(int kind, const void *dy, const uint8_t *argmax, const void *y, void *dx, float *db,
                          int N, int C, int H, int W, int k, int d, dsk_act act, dsk_dtype t,
                          void *ws, size_t ws_bytes, void *stream)
{
    if (kind != DSK_MAXPOOL && kind != DSK_AVGPOOL) return DSK_EINVAL;
    int rc = pool_check(dy, dx, N, C, H, W, k, d, t);
    if (rc != DSK_OK) return rc;
    if (kind == DSK_MAXPOOL && bad_ptr(argmax)) return DSK_EINVAL;
    if (act < DSK_ACT_NONE || act > DSK_ACT_TANH || bad_ptr(db)) return DSK_EINVAL;
    if (act != DSK_ACT_NONE && bad_ptr(y)) return DSK_EINVAL;
    const size_t need = dsk_pool_bwd_act_bias_workspace_bytes(kind, N, C, H, W, k, d, t);
    if (ws == nullptr || !aligned16(ws) || ws_bytes < need) return DSK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    clear_errors();
    if (pool_walk_ok(N, C, H, W, k, d, t))
        return launch_pool_walk_bwd(dy, argmax, dx, y, db, act, ws, N, C, H, W, k, d, kind == DSK_MAXPOOL, t, st);
    // other window sizes: the two passes one after the other
    rc = kind == DSK_MAXPOOL ? launch_maxpool_bwd(dy, argmax, dx, N, C, H, W, k, d, t, st)
                             : launch_avgpool_bwd(dy, dx, N, C, H, W, k, d, t, st);
    if (rc != DSK_OK) return rc;
    return launch_act_bwd_bias(y, dx, db, N, C, (long)H * W, act, t, ws, st);
}

int dsk_act_bwd(const void *y, void *dy, size_t count, dsk_act act, dsk_dtype t, void *stream)
{
    if (bad_ptr(y) || bad_ptr(dy) || bad_dtype(t)) return DSK_EINVAL;
    if (act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    if (count > (size_t)kMaxElems) return DSK_ESHAPE;
    clear_errors();
    return launch_act_bwd(y, dy, count, act, t, (hipStream_t)stream);
}

size_t dsk_act_bwd_bias_workspace_bytes(int K)
{
    return K < 1 ? 0 : act_bwd_bias_ws_bytes(K);
}

int dsk_act_bwd_bias(const void *y, void *dy, float *db, int N, int K, int Ho, int Wo, dsk_act act, dsk_dtype t,
                     void *ws, size_t ws_bytes, void *stream)
{
    if (bad_ptr(dy) || bad_ptr(db) || bad_dtype(t)) return DSK_EINVAL;
    if (act < DSK_ACT_NONE || act > DSK_ACT_TANH) return DSK_EINVAL;
    if (act != DSK_ACT_NONE && bad_ptr(y)) return DSK_EINVAL;
    if (N < 1 || K < 1 || Ho < 1 || Wo < 1) return DSK_EINVAL;
    if ((long)N * K * Ho * Wo > kMaxElems) return DSK_ESHAPE;
    if (ws == nullptr || !aligned16(ws) || ws_bytes < act_bwd_bias_ws_bytes(K)) return DSK_EWORKSPACE;
    clear_errors();
    return launch_act_bwd_bias(y, dy, db, N, K, (long)Ho * Wo, act, t, ws, (hipStream_t)stream);
}

size_t dsk_softmax_xent_workspace_bytes(int N, int Cls, int H, int W)
{
    if (N < 1 || Cls < 1 || H < 1 || W < 1) return 0;
    return softmax_xent_ws_bytes((long)N * H * W);
}

int dsk_masked_softmax_xent(const float *scores, const int32_t *labels, const uint8_t *mask,
                            float *loss, void *dscores, dsk_dtype dt, int N, int Cls, int H, int W,
                            void *ws, size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt)) return DSK_EINVAL;
    if (bad_ptr(scores) || bad_ptr(labels) || bad_ptr(mask) || bad_ptr(dscores) || loss == nullptr ||
        (reinterpret_cast<uintptr_t>(loss) & 3u))
        return DSK_EINVAL;
    if (N < 1 || Cls < 1 || H < 1 || W < 1) return DSK_EINVAL;
    if ((long)N * Cls * H * W > kMaxElems) return DSK_ESHAPE;
    const size_t need = softmax_xent_ws_bytes((long)N * H * W);
    if (ws == nullptr || !aligned16(ws) || ws_bytes < need) return DSK_EWORKSPACE;
    clear_errors();
    return launch_masked_softmax_xent(scores, labels, mask, loss, dscores, dt, N, Cls, H, W, ws, (hipStream_t)stream);
}

int dsk_masked_softmax_xent_static(const float *scores, const int32_t *labels, const uint8_t *mask,
                                   float *loss, void *dscores, dsk_dtype dt, int N, int Cls, int H, int W,
                                   void *stream)
{
    if (bad_dtype(dt)) return DSK_EINVAL;
    if (bad_ptr(scores) || bad_ptr(labels) || bad_ptr(mask) || bad_ptr(dscores) || loss == nullptr ||
        (reinterpret_cast<uintptr_t>(loss) & 3u))
        return DSK_EINVAL;
    if (N < 1 || Cls < 1 || H < 1 || W < 1) return DSK_EINVAL;
    if ((long)N * Cls * H * W > kMaxElems) return DSK_ESHAPE;
    void *ws = nullptr;
    const int rc = static_scratch_of_current_device(&ws);
    if (rc != DSK_OK) return rc;
    clear_errors();
    return launch_masked_softmax_xent(scores, labels, mask, loss, dscores, dt, N, Cls, H, W, ws, (hipStream_t)stream);
}

} // extern "C"
