/*
 * libdsk -- whole-image forward / backward propagation of a patch-classification
 * CNN with d-regularly sparse kernels, for AMD MI355X (gfx950).
 *
 * Every stride-s convolution, pooling and fully connected layer of the original
 * patch CNN becomes a stride-1 layer whose k x k kernel has its neighbouring
 * entries d pixels apart (paper Sec. 3.2); Algorithm 1 gives d per layer.  One
 * pass over the padded image then yields, at every pixel, what the original CNN
 * yields on the patch around that pixel, and one backward pass with a pixel mask
 * on the last error map yields the summed gradients of the masked patches
 * (Sec. 4).  The zeros of the sparse kernels are never stored or multiplied: a
 * layer is described by its dense k x k kernel and the spacing d.
 *
 * Conventions (all entry points unless stated otherwise)
 *   - Tensors are dense, row-major NCHW (W fastest).  H, W in a call are the
 *     INPUT map's size; the output is Ho = H-(kh-1)*d by Wo = W-(kw-1)*d.
 *   - Pointers are DEVICE pointers owned by the caller, base-aligned to 16 bytes.
 *     The library never allocates, frees, copies to the host or synchronises; all
 *     work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default).
 *   - Outputs are overwritten.  Inputs and outputs must not alias unless stated.
 *   - Weights w[K][C][kh][kw], bias b[K], their gradients, the loss and the last
 *     error map are always fp32.  `in` / `out` / `t` give the type of the
 *     activation tensors: DSK_F32, or DSK_BF16 (bfloat16 storage; products are
 *     accumulated in fp32, weights are rounded to bf16 inside the kernel).
 *   - Arguments are validated before anything is launched, so every error below
 *     except DSK_ELAUNCH is returned without touching the GPU.  No exceptions
 *     cross this boundary.  Calls are re-entrant: the library keeps no state
 *     between calls apart from the calling thread's diagnostic switch
 *     dsk_set_conv_algo and the per-GPU scratch array of
 *     dsk_masked_softmax_xent_static.
 *   - Return value: DSK_OK (0) or a negative dsk_status.
 */
#ifndef DSK_H
#define DSK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DSK_OK = 0,
    DSK_EINVAL = -1,     /* null / misaligned pointer, N,C,K,k < 1, d < 1, bad enum value   */
    DSK_ESHAPE = -2,     /* output would be empty, k*k > 255 (pool), tensor over 2^31-1 elements */
    DSK_EDTYPE = -3,     /* dtype combination not supported by this entry point            */
    DSK_EWORKSPACE = -4, /* workspace NULL or smaller than dsk_*_workspace_bytes says      */
    DSK_ELAUNCH = -5     /* the HIP runtime reported an error at launch                    */
} dsk_status;

typedef enum { DSK_F32 = 0, DSK_BF16 = 1 } dsk_dtype;
typedef enum { DSK_ACT_NONE = 0, DSK_ACT_RELU = 1, DSK_ACT_TANH = 2 } dsk_act;
typedef enum { DSK_CONV = 0, DSK_MAXPOOL = 1, DSK_AVGPOOL = 2 } dsk_kind;

/* ------------------------------------------------------------------------- */
/* Host-side planner: Algorithm 1's bookkeeping.  HOST pointers, no GPU use.   */
/* ------------------------------------------------------------------------- */

/* One layer of the ORIGINAL strided patch CNN.  A fully connected layer is a
 * conv whose kernel covers the whole remaining map (Sec. 3.4, last paragraph). */
typedef struct {
    int kind; /* dsk_kind */
    int K;    /* conv: output channels; pools: ignored */
    int k;    /* square kernel size */
    int s;    /* stride in the original CNN */
    int act;  /* conv: dsk_act applied to the output */
} dsk_layer;

/* The same layer in the whole-image network: stride 1, kernel spacing d. */
typedef struct {
    int kind, act;
    int C, K;         /* input / output channels */
    int k, d;         /* kernel size and spacing (Algorithm 1: d = product of earlier strides) */
    int H, W;         /* input map size */
    int Ho, Wo;       /* output map size = H-(k-1)*d, W-(k-1)*d */
} dsk_layer_plan;

/* Algorithm 1 for an image of H x W pixels with C0 channels.  Fills out[0..L-1].
 *   *rf       receptive field 1 + sum (k-1)*d: the patch size for which the
 *             original CNN ends in a 1 x 1 map when all its strides divide evenly
 *   n         declared patch size of the original CNN, or 0 to use *rf.  n > *rf
 *             (strides that do not divide evenly: the original CNN ignores the
 *             trailing rows/columns of its patch) is allowed, n < *rf is DSK_ESHAPE
 *   *pad_lo   zero rows/columns to add on the top/left  = floor(n/2)      (Sec. 3.3)
 *   *pad_hi   ... on the bottom/right = *rf - 1 - *pad_lo, so that the padded
 *             image is (H + *rf - 1) x (W + *rf - 1) and the last map is H x W
 * Any of rf / pad_lo / pad_hi may be NULL.  Errors: DSK_EINVAL, DSK_ESHAPE. */
int dsk_plan(const dsk_layer *layers, int L, int C0, int H, int W, int n,
             dsk_layer_plan *out, int *rf, int *pad_lo, int *pad_hi);

const char *dsk_status_string(int status);

/* ------------------------------------------------------------------------- */
/* Image padding (Sec. 3.3): once, at the input only.                          */
/* ------------------------------------------------------------------------- */

/* xpad[N][C][H+lo+hi][W+lo+hi] (type `out`) = zero-padded copy of the fp32 image
 * x[N][C][H][W]: lo zero rows/columns on the top/left, hi on the bottom/right. */
int dsk_pad_image(const float *x, void *xpad, int N, int C, int H, int W,
                  int lo, int hi, dsk_dtype out, void *stream);

/* ------------------------------------------------------------------------- */
/* Stride-1 convolution with a d-regularly sparse kernel (Sec. 3.1-3.2, Alg. 1) */
/* ------------------------------------------------------------------------- */

typedef enum { DSK_WS_CONV_FWD = 0, DSK_WS_CONV_BWD_DATA = 1, DSK_WS_CONV_BWD_WEIGHT = 2 } dsk_ws_which;

/* Bytes of scratch device memory the matching conv call needs (0 is possible). */
size_t dsk_conv_workspace_bytes(int which, int N, int C, int H, int W, int K,
                                int kh, int kw, int d, dsk_dtype in);

/* Forward, y_k = W_{k,d} *^1 x_k + b_k followed by the non-linearity:
 *   y[n][f][u][v] = act( b[f] + sum_{c,a,b} w[f][c][a][b] * x[n][c][u+a*d][v+b*d] )
 * x[N][C][H][W] (`in`), y[N][K][Ho][Wo] (`out`), b may be NULL (no bias). */
int dsk_conv_fwd(const void *x, const float *w, const float *b, void *y,
                 int N, int C, int H, int W, int K, int kh, int kw, int d,
                 dsk_dtype in, dsk_dtype out, dsk_act act,
                 void *ws, size_t ws_bytes, void *stream);

/* Error map of the layer's input (Sec. 4.1): delta_k = pad(delta_{k+1}) *^1 rot180(W_{k,d}),
 *   dx[n][c][p][q] = sum_{f,a,b} dy[n][f][p-a*d][q-b*d] * w[f][c][a][b]   (dy = 0 outside its map)
 * dy[N][K][Ho][Wo] (`in`), dx[N][C][H][W] (`out`). */
int dsk_conv_bwd_data(const void *dy, const float *w, void *dx,
                      int N, int C, int H, int W, int K, int kh, int kw, int d,
                      dsk_dtype in, dsk_dtype out,
                      void *ws, size_t ws_bytes, void *stream);

/* Gradients of the non-zero kernel entries and of the bias (Sec. 4.1):
 *   dw[f][c][a][b] = sum_{n,u,v} dy[n][f][u][v] * x[n][c][u+a*d][v+b*d]
 *   db[f]          = sum_{n,u,v} dy[n][f][u][v]                       (db may be NULL)
 * x and dy have type `in`; dw, db are fp32.  The summation order is fixed: two
 * calls on the same input give bit-identical results. */
int dsk_conv_bwd_weight(const void *x, const void *dy, float *dw, float *db,
                        int N, int C, int H, int W, int K, int kh, int kw, int d,
                        dsk_dtype in, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Stride-1 pooling with a d-regularly sparse k x k kernel (Sec. 3.1-3.2, 4.2)  */
/* ------------------------------------------------------------------------- */

/* y[n][c][u][v] = max_{a,b} x[n][c][u+a*d][v+b*d]; argmax[n][c][u][v] = a*k+b of the
 * winner ("the index within every patch", Sec. 4.2).  Taps are visited in the
 * order a*k+b and replace the running maximum only when strictly greater, so the
 * lowest index wins ties (and -0.0 == +0.0).  NaN inputs are unsupported.
 * argmax may be NULL (inference).  Needs k*k <= 255. */
int dsk_maxpool_fwd(const void *x, void *y, uint8_t *argmax,
                    int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream);

/* Errors accumulate at the recorded locations (Sec. 4.2):
 *   dx[n][c][p][q] = sum_{a,b} [argmax[n][c][p-a*d][q-b*d] == a*k+b] * dy[n][c][p-a*d][q-b*d]
 * Gather form, fixed summation order, no atomics. */
int dsk_maxpool_bwd(const void *dy, const uint8_t *argmax, void *dx,
                    int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream);

/* y = mean of the k*k taps (divisor always k*k: no padding exists inside the net). */
int dsk_avgpool_fwd(const void *x, void *y,
                    int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream);

/* dx[n][c][p][q] = (1/k^2) sum_{a,b} dy[n][c][p-a*d][q-b*d]: a mean filter (Sec. 4.2). */
int dsk_avgpool_bwd(const void *dy, void *dx,
                    int N, int C, int H, int W, int k, int d, dsk_dtype t, void *stream);

/* ------------------------------------------------------------------------- */
/* Point-wise non-linearity, backward (Sec. 1: the non-linearity layer)        */
/* ------------------------------------------------------------------------- */

/* In place: dy[i] *= act'(.) expressed through the layer's OUTPUT y:
 * ReLU: [y > 0];  tanh: 1 - y*y;  none: no-op.  y and dy have type t. */
int dsk_act_bwd(const void *y, void *dy, size_t count, dsk_act act, dsk_dtype t, void *stream);

/* The same, fused with the bias gradient of the conv layer that produced y (Sec. 4.1: the
 * gradient of b_k is the sum of all entries of the error map), in one pass over the map:
 *   dy[n][f][u][v] *= act'(.)   in place (act = DSK_ACT_NONE leaves dy untouched, y may be NULL)
 *   db[f] = sum_{n,u,v} dy[n][f][u][v]   of the values as stored back (fp32, fixed order)
 * dy[N][K][Ho][Wo] and y have type t.  A caller that uses this passes db = NULL to
 * dsk_conv_bwd_weight.  Workspace: dsk_act_bwd_bias_workspace_bytes(K). */
size_t dsk_act_bwd_bias_workspace_bytes(int K);
int dsk_act_bwd_bias(const void *y, void *dy, float *db, int N, int K, int Ho, int Wo,
                     dsk_act act, dsk_dtype t, void *ws, size_t ws_bytes, void *stream);

/* A pooling layer's gradient fused with the backward of the convolution layer in front of it, in ONE pass
 * over the error map (Sec. 4.2 for the pool; Sec. 1 / Sec. 4.1 for the non-linearity and the bias):
 *   dx[n][c][p][q] = act'(.) * (pool gradient of dy at [n][c][p][q])   act' through that layer's output y
 *   db[c]          = sum_{n,p,q} dx[n][c][p][q]   of the values as stored (fp32, fixed order)
 * kind: DSK_MAXPOOL (argmax as recorded by dsk_maxpool_fwd) or DSK_AVGPOOL (argmax ignored, may be NULL).
 * dy[N][C][Ho][Wo], y and dx [N][C][H][W], all of type t; y may be NULL for DSK_ACT_NONE.  The result equals
 * dsk_maxpool_bwd / dsk_avgpool_bwd followed by dsk_act_bwd_bias: dx is then the error map that
 * dsk_conv_bwd_weight (with db = NULL) and dsk_conv_bwd_data of the convolution layer take. */
size_t dsk_pool_bwd_act_bias_workspace_bytes(int kind, int N, int C, int H, int W, int k, int d, dsk_dtype t);
int dsk_pool_bwd_act_bias(int kind, const void *dy, const uint8_t *argmax, const void *y, void *dx, float *db,
                          int N, int C, int H, int W, int k, int d, dsk_act act, dsk_dtype t,
                          void *ws, size_t ws_bytes, void *stream);

/* A convolution layer's backward-data fused with the backward of the convolution layer directly below it
 * (no pool in between, e.g. the two fully connected layers at the top of a network), Sec. 4.1:
 *   dx[n][c][p][q] = act'(.) * (dsk_conv_bwd_data of dy and w at [n][c][p][q])   act' through x
 *   db[c]          = sum_{n,p,q} dx[n][c][p][q]   of the values as stored (fp32, fixed order)
 * x[N][C][H][W] is this layer's input, i.e. the stored output of the layer below, whose non-linearity is
 * `act` and whose bias gradient is db; x and dx have type `out`; x may be NULL for DSK_ACT_NONE.  The result
 * equals dsk_conv_bwd_data followed by dsk_act_bwd_bias(x, dx, db, N, C, H, W, act, out).  1 x 1 kernels with
 * in == out write the error map once, from the epilogue of the matrix kernel; every other shape runs the two
 * passes one after the other.  db is required; a caller that uses this passes db = NULL to dsk_conv_bwd_weight
 * of the layer below.  Workspace: dsk_conv_bwd_data_act_bias_workspace_bytes (enough for either form; 0 for an
 * invalid shape).  Errors as for dsk_conv_bwd_data; the summation order is fixed (bit-identical repeats). */
size_t dsk_conv_bwd_data_act_bias_workspace_bytes(int N, int C, int H, int W, int K, int kh, int kw, int d,
                                                  dsk_dtype in, dsk_dtype out);
int dsk_conv_bwd_data_act_bias(const void *dy, const float *w, const void *x, void *dx, float *db,
                               int N, int C, int H, int W, int K, int kh, int kw, int d,
                               dsk_dtype in, dsk_dtype out, dsk_act act,
                               void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Last layer: masked softmax cross-entropy (pixel mask of Sec. 4.3)           */
/* ------------------------------------------------------------------------- */

size_t dsk_softmax_xent_workspace_bytes(int N, int Cls, int H, int W);

/* scores[N][Cls][H][W] fp32, labels[N][H][W] int32 in [0, Cls), mask[N][H][W] u8.
 *   p       = softmax over classes at each pixel (row maximum subtracted)
 *   count   = number of pixels with mask != 0 in the whole batch
 *   loss[0] = -(1/count) * sum_{mask != 0} log p[label]        (0 if count == 0)
 *   dscores = (mask != 0) * (p - onehot(label)) / count        (0 if count == 0)
 *             [N][Cls][H][W], stored in type `dt` (the arithmetic is fp32 either way)
 * Errors of unchosen pixels are exactly zero (they are written without their
 * scores being read, so the call gets a little cheaper as the mask gets sparser;
 * everything after it in the backward pass is dense, Sec. 4.3).
 * A label outside [0, Cls) at a chosen pixel is the caller's error (the pixel
 * then contributes p as its error and nothing to the loss).  loss: 1 device float. */
int dsk_masked_softmax_xent(const float *scores, const int32_t *labels, const uint8_t *mask,
                            float *loss, void *dscores, dsk_dtype dt, int N, int Cls, int H, int W,
                            void *ws, size_t ws_bytes, void *stream);

/* The same call for callers that cannot allocate device memory or size a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments and results as dsk_masked_softmax_xent
 * minus the workspace: the partial counts and sums live in an array the
 * library holds in every GPU's memory until the process ends (8208 bytes:
 * 1024 counts and 1024 sums, whatever the size of the map).
 *   - Size limits are those of dsk_masked_softmax_xent (N*Cls*H*W <= 2^31-1,
 *     else DSK_ESHAPE): the scratch array never is what limits a call.
 *   - The device of `stream` must be the current device.  The first call on a
 *     device looks the array up (no allocation); make it outside graph capture.
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one
 *     GPU (different streams, different threads) race.  The array is re-initialised
 *     by each call's own kernels, so nothing has to be cleared in between. */
int dsk_masked_softmax_xent_static(const float *scores, const int32_t *labels, const uint8_t *mask,
                                   float *loss, void *dscores, dsk_dtype dt, int N, int Cls, int H, int W,
                                   void *stream);

/* ------------------------------------------------------------------------- */
/* Fast scanning: the method the paper compares with (Sec. 2; Sec. 3.6, last    */
/* paragraph; Table 1).  Forward only.  A comparator, not part of the hot path. */
/* ------------------------------------------------------------------------- */

/* Fast scanning keeps every layer's ORIGINAL stride s and runs a strided layer s*s times, once per
 * starting offset (ay, ax); every run yields one output fragment.  With fragment spacing D (the product of
 * the strides so far) an image has D*D fragments, stored as a batch [N*D*D][C][h][w] with index
 * n*D*D + fy*D + fx: fragment (fy, fx) holds the whole-image map's entries (fy + D*u, fx + D*v); all
 * fragments have the size of the largest one, h = ceil(H/D), smaller ones leave their last row / column
 * unused.  Stride-1 layers are ordinary dense layers on that batch (dsk_conv_fwd with d = 1).
 *
 * dsk_fs_pool_fwd / dsk_fs_conv_fwd: one strided layer, all s*s offsets in one call:
 *   out fragment (fy + D*ay, fx + D*ax) at spacing D*s, entry (u, v)
 *       = pool / conv of in fragment (fy, fx) over the taps (ay + s*u + a, ax + s*v + b), 0 <= a, b < k
 * in[N*D*D][C][hi][wi], out[N*D*s*D*s][C or K][ho][wo]; taps outside the stored fragment are skipped (they
 * only ever belong to entries that are unused themselves).  One thread per output entry, taps read at
 * stride s with the run's offset: that access pattern is the method.
 * dsk_fs_assemble: the label map out[n][c][i][j] = fragment (n, i % D, j % D), entry (i / D, j / D). */
int dsk_fs_pool_fwd(int kind, const void *in, void *out, int N, int D, int C, int hi, int wi, int k, int s,
                    int ho, int wo, dsk_dtype t, void *stream);
int dsk_fs_conv_fwd(const void *in, const float *w, const float *b, void *out, int N, int D, int C, int hi, int wi,
                    int K, int k, int s, int ho, int wo, dsk_act act, dsk_dtype t, void *stream);
int dsk_fs_assemble(const void *frag, void *out, int N, int D, int C, int hf, int wf, int H, int W,
                    dsk_dtype tin, dsk_dtype tout, void *stream);

/* ------------------------------------------------------------------------- */
/* Video: 3-D convolution and 3-D pooling with kernels sparse in time and space  */
/* (Sec. 6 proposes carrying the method over to video; Sec. 3.1-3.2, Sec. 4 and   */
/* Algorithm 1 applied to the temporal axis as well)                           */
/* ------------------------------------------------------------------------- */

/* A cube classifier (nt frames of n x n pixels per labelled voxel) with temporal strides st and spatial
 * strides s becomes a stride-1 network over the whole padded video: layer k's kernel has its temporal
 * taps dt frames apart and its spatial taps d pixels apart, where dt / d are the products of the earlier
 * temporal / spatial strides (dsk_plan on the (kt, st) list gives dt, on the (k, s) list gives d).
 *
 * Layout: maps [N][T][C][H][W] (frame-major: a video is a batch of T images, so dsk_pad_image,
 * dsk_act_bwd*, dsk_masked_softmax_xent apply with N*T images); weights w[kt][K][C][kh][kw] fp32
 * (one 2-D kernel per temporal tap), bias [K].  Output: [N][To][K][Ho][Wo], To = T-(kt-1)*dt,
 * Ho = H-(kh-1)*d, Wo = W-(kw-1)*d.  All pointers are device pointers, 16-byte aligned; nothing is
 * allocated; errors as for the 2-D calls.  kt = 1 is the 2-D layer applied to every frame.
 *
 *   y[n][t][f][u][v]  = act( b[f] + sum_{e,c,a,b} w[e][f][c][a][b] * x[n][t+e*dt][c][u+a*d][v+b*d] )
 *   dx[n][t][c][p][q] = sum_{e,f,a,b} dy[n][t-e*dt][f][p-a*d][q-b*d] * w[e][f][c][a][b]   (dy = 0 outside)
 *   dw[e][f][c][a][b] = sum_{n,t,u,v} dy[n][t][f][u][v] * x[n][t+e*dt][c][u+a*d][v+b*d]
 *   db[f]             = sum_{n,t,u,v} dy[n][t][f][u][v]                    (db may be NULL) */
/* xpad[N][T+tlo+thi][C][H+lo+hi][W+lo+hi] (type `out`) = zero-padded copy of the fp32 video x[N][T][C][H][W]:
 * tlo / thi zero frames before / after, lo / hi zero rows and columns (Sec. 3.3 on all three axes). */
int dsk_pad_video(const float *x, void *xpad, int N, int T, int C, int H, int W,
                  int tlo, int thi, int lo, int hi, dsk_dtype out, void *stream);

size_t dsk_conv3d_workspace_bytes(int which, int N, int T, int C, int H, int W, int K,
                                  int kt, int kh, int kw, int dt, int d, dsk_dtype in);
int dsk_conv3d_fwd(const void *x, const float *w, const float *b, void *y,
                   int N, int T, int C, int H, int W, int K, int kt, int kh, int kw, int dt, int d,
                   dsk_dtype in, dsk_dtype out, dsk_act act, void *ws, size_t ws_bytes, void *stream);
int dsk_conv3d_bwd_data(const void *dy, const float *w, void *dx,
                        int N, int T, int C, int H, int W, int K, int kt, int kh, int kw, int dt, int d,
                        dsk_dtype in, dsk_dtype out, void *ws, size_t ws_bytes, void *stream);
int dsk_conv3d_bwd_weight(const void *x, const void *dy, float *dw, float *db,
                          int N, int T, int C, int H, int W, int K, int kt, int kh, int kw, int dt, int d,
                          dsk_dtype in, void *ws, size_t ws_bytes, void *stream);

/* 3-D pooling over kt x k x k taps (dt frames, d pixels apart); x[N][T][C][H][W] -> y[N][To][C][Ho][Wo].
 * Max pooling records the winner's index (e*k + a)*k + b (needs kt*k*k <= 255); taps are visited in that
 * order and replace the maximum only when strictly greater, so the lowest index wins ties.  Backward is the
 * gather form of Sec. 4.2 (fixed order, no atomics); the average pool divides by kt*k*k.  argmax may be
 * NULL in dsk_maxpool3d_fwd. */
int dsk_maxpool3d_fwd(const void *x, void *y, uint8_t *argmax, int N, int T, int C, int H, int W,
                      int kt, int k, int dt, int d, dsk_dtype t, void *stream);
int dsk_maxpool3d_bwd(const void *dy, const uint8_t *argmax, void *dx, int N, int T, int C, int H, int W,
                      int kt, int k, int dt, int d, dsk_dtype t, void *stream);
int dsk_avgpool3d_fwd(const void *x, void *y, int N, int T, int C, int H, int W,
                      int kt, int k, int dt, int d, dsk_dtype t, void *stream);
int dsk_avgpool3d_bwd(const void *dy, void *dx, int N, int T, int C, int H, int W,
                      int kt, int k, int dt, int d, dsk_dtype t, void *stream);

/* ------------------------------------------------------------------------- */
/* Kernel selection (diagnostics)                                              */
/* ------------------------------------------------------------------------- */

/* 0 = automatic (matrix-core kernels where they apply), 1 = force the plain
 * one-thread-per-output kernels, 2 = automatic but bf16 maps are multiplied on the
 * fp32 matrix path (converted while they are staged) instead of the bf16 one.
 * Applies to the calling thread's later calls only; returns the previous value
 * (an invalid argument changes nothing). */
int dsk_set_conv_algo(int algo);

#ifdef __cplusplus
}
#endif
#endif /* DSK_H */
