/*
 * TEST INFRASTRUCTURE -- the CPU oracle.  Not part of the product: only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Literal patch-by-patch scanning (paper Sec. 1.1 and Fig. 1(a)): for every
 * requested pixel the n x n patch is cropped from the padded image and pushed
 * through the ORIGINAL strided CNN; backward feeds each patch's output error
 * through the textbook backward pass of that CNN and sums the per-patch
 * parameter gradients (Sec. 4.3: the whole-image gradients with a mask equal
 * those of the mini-batch of masked patches through the original CNN).
 *
 * Nothing here knows about dilation / d-regularly sparse kernels: that is the
 * method under test.  All arithmetic is fp64, plain nested loops, no blocking.
 *
 * Layers of the original CNN ("valid", no per-layer padding):
 *   conv    y[k][u][v] = act(b[k] + sum_{c,a,b} w[k][c][a][b] x[c][u*s+a][v*s+b])
 *           (cross-correlation, Sec. 3.1: y_k = W_k *^{d_k} x_k + b_k)
 *   maxpool y[c][u][v] = max_{a,b} x[c][u*s+a][v*s+b]; the index a*k+b of the
 *           winning tap is recorded (Sec. 4.2); taps are scanned row-major and
 *           replaced only on strict '>', so the lowest index wins ties
 *   avgpool y[c][u][v] = (1/k^2) sum_{a,b} x[c][u*s+a][v*s+b]
 * Output size (m-k)/s+1 with floor.  A fully connected layer is a conv whose
 * kernel spans the whole remaining map (Sec. 3.4).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_CONV = 0, ORC_MAXPOOL = 1, ORC_AVGPOOL = 2 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1, ORC_ACT_TANH = 2 };

typedef struct {
    int kind; /* ORC_CONV / ORC_MAXPOOL / ORC_AVGPOOL */
    int K;    /* conv: output channels */
    int k;    /* kernel size (square) */
    int s;    /* stride */
    int act;  /* conv: ORC_ACT_* */
} orc_layer;

#define ORC_MAX_LAYERS 64

typedef struct {
    int nL;
    int C[ORC_MAX_LAYERS + 1];       /* channels of map l (map 0 = input patch) */
    int m[ORC_MAX_LAYERS + 1];       /* spatial size of map l */
    long act_off[ORC_MAX_LAYERS + 2];/* offset of map l in the activation buffer */
    long par_off[ORC_MAX_LAYERS + 1];/* offset of layer l's weights in params (conv only) */
    long n_params;
} orc_geom;

static int geom_build(const orc_layer *L, int nL, int C0, int n, orc_geom *g)
{
    if (nL < 1 || nL > ORC_MAX_LAYERS || C0 < 1 || n < 1) return -1;
    g->nL = nL;
    g->C[0] = C0;
    g->m[0] = n;
    g->act_off[0] = 0;
    long po = 0;
    for (int l = 0; l < nL; ++l) {
        if (L[l].k < 1 || L[l].s < 1 || L[l].k > g->m[l]) return -1;
        g->m[l + 1] = (g->m[l] - L[l].k) / L[l].s + 1;
        g->act_off[l + 1] = g->act_off[l] + (long)g->C[l] * g->m[l] * g->m[l];
        g->par_off[l] = po;
        if (L[l].kind == ORC_CONV) {
            if (L[l].K < 1) return -1;
            g->C[l + 1] = L[l].K;
            po += (long)L[l].K * g->C[l] * L[l].k * L[l].k + L[l].K;
        } else if (L[l].kind == ORC_MAXPOOL || L[l].kind == ORC_AVGPOOL) {
            g->C[l + 1] = g->C[l];
        } else {
            return -1;
        }
    }
    g->act_off[nL + 1] = g->act_off[nL] + (long)g->C[nL] * g->m[nL] * g->m[nL];
    g->n_params = po;
    return 0;
}

/* Sizes a caller needs: total activation doubles for one patch (all maps,
 * input included), parameter count, class count, final spatial size. */
int orc_sizes(const orc_layer *L, int nL, int C0, int n,
              long *act_total, long *n_params, int *classes, int *m_last)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g)) return -1;
    if (act_total) *act_total = g.act_off[nL + 1];
    if (n_params) *n_params = g.n_params;
    if (classes) *classes = g.C[nL];
    if (m_last) *m_last = g.m[nL];
    return 0;
}

/* Per-map geometry: C[l], m[l], act_off[l] for l = 0..nL, par_off[l] for l < nL. */
int orc_geometry(const orc_layer *L, int nL, int C0, int n,
                 int *C, int *m, long *act_off, long *par_off)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g)) return -1;
    for (int l = 0; l <= nL; ++l) { C[l] = g.C[l]; m[l] = g.m[l]; act_off[l] = g.act_off[l]; }
    for (int l = 0; l < nL; ++l) par_off[l] = g.par_off[l];
    return 0;
}

static double act_apply(int act, double z)
{
    if (act == ORC_ACT_RELU) return z > 0.0 ? z : 0.0;
    if (act == ORC_ACT_TANH) return tanh(z);
    return z;
}

/* derivative of the activation expressed through its output y */
static double act_grad_from_output(int act, double y)
{
    if (act == ORC_ACT_RELU) return y > 0.0 ? 1.0 : 0.0;
    if (act == ORC_ACT_TANH) return 1.0 - y * y;
    return 1.0;
}

/* Storage precision of the maps.  ORC_STORE_EXACT keeps every value in fp64.
 * ORC_STORE_BF16 models a path that STORES activations in bfloat16: the patch and
 * every layer output except the last are rounded to bfloat16 (nearest even) after
 * being computed in fp64, so that the decisions taken on stored values (ReLU
 * gates, max-pool winners) are taken in the storage precision. */
enum { ORC_STORE_EXACT = 0, ORC_STORE_BF16 = 1 };

static double round_bf16(double v)
{
    union { float f; unsigned u; } c;
    c.f = (float)v;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) return v; /* NaN */
    c.u += 0x7fffu + ((c.u >> 16) & 1u);
    c.u &= 0xffff0000u;
    return (double)c.f;
}

static void round_map(double *p, long count, int storage)
{
    if (storage == ORC_STORE_BF16)
        for (long t = 0; t < count; ++t) p[t] = round_bf16(p[t]);
}

/* Forward of the original CNN on one patch.  acts[act_off[0]...] must already
 * hold the patch (C0 x n x n).  Fills every later map; amax gets, at the same
 * offsets as the map it belongs to, the winning tap index of each max-pool
 * output (other entries untouched).  pre (may be NULL) gets, at the offsets of
 * each conv layer's output map, the value BEFORE the non-linearity (bias
 * included); entries of other maps are untouched. */
static void patch_forward(const orc_layer *L, const orc_geom *g, const double *params,
                          double *acts, int *amax, int storage, double *pre)
{
    round_map(acts + g->act_off[0], g->act_off[1] - g->act_off[0], storage);
    for (int l = 0; l < g->nL; ++l) {
        const int Ci = g->C[l], mi = g->m[l], Co = g->C[l + 1], mo = g->m[l + 1];
        const int k = L[l].k, s = L[l].s;
        const double *x = acts + g->act_off[l];
        double *y = acts + g->act_off[l + 1];
        if (L[l].kind == ORC_CONV) {
            const double *w = params + g->par_off[l];
            const double *b = w + (long)Co * Ci * k * k;
            double *z = pre ? pre + g->act_off[l + 1] : NULL;
            for (int f = 0; f < Co; ++f)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        double acc = b[f];
                        for (int c = 0; c < Ci; ++c)
                            for (int a = 0; a < k; ++a)
                                for (int bb = 0; bb < k; ++bb)
                                    acc += w[(((long)f * Ci + c) * k + a) * k + bb] *
                                           x[((long)c * mi + (u * s + a)) * mi + (v * s + bb)];
                        y[((long)f * mo + u) * mo + v] = act_apply(L[l].act, acc);
                        if (z) z[((long)f * mo + u) * mo + v] = acc;
                    }
        } else if (L[l].kind == ORC_MAXPOOL) {
            int *am = amax ? amax + g->act_off[l + 1] : NULL;
            for (int c = 0; c < Ci; ++c)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        double best = x[((long)c * mi + u * s) * mi + v * s];
                        int bi = 0;
                        for (int a = 0; a < k; ++a)
                            for (int bb = 0; bb < k; ++bb) {
                                double t = x[((long)c * mi + (u * s + a)) * mi + (v * s + bb)];
                                if (t > best) { best = t; bi = a * k + bb; }
                            }
                        y[((long)c * mo + u) * mo + v] = best;
                        if (am) am[((long)c * mo + u) * mo + v] = bi;
                    }
        } else { /* ORC_AVGPOOL */
            for (int c = 0; c < Ci; ++c)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        double acc = 0.0;
                        for (int a = 0; a < k; ++a)
                            for (int bb = 0; bb < k; ++bb)
                                acc += x[((long)c * mi + (u * s + a)) * mi + (v * s + bb)];
                        y[((long)c * mo + u) * mo + v] = acc / (double)(k * k);
                    }
        }
        if (l + 1 < g->nL) round_map(y, (long)Co * mo * mo, storage);
    }
}

/* Textbook backward of the original CNN on one patch.  grads holds, at the
 * offsets of each map, dLoss/dmap; the entry for the last map must be filled
 * by the caller, all earlier ones must be zero.  dparams is accumulated. */
static void patch_backward(const orc_layer *L, const orc_geom *g, const double *params,
                           const double *acts, const int *amax, double *grads, double *dparams)
{
    for (int l = g->nL - 1; l >= 0; --l) {
        const int Ci = g->C[l], mi = g->m[l], Co = g->C[l + 1], mo = g->m[l + 1];
        const int k = L[l].k, s = L[l].s;
        const double *x = acts + g->act_off[l];
        const double *y = acts + g->act_off[l + 1];
        const double *dy = grads + g->act_off[l + 1];
        double *dx = grads + g->act_off[l];
        if (L[l].kind == ORC_CONV) {
            const double *w = params + g->par_off[l];
            double *dw = dparams + g->par_off[l];
            double *db = dw + (long)Co * Ci * k * k;
            for (int f = 0; f < Co; ++f)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        const long o = ((long)f * mo + u) * mo + v;
                        const double dz = dy[o] * act_grad_from_output(L[l].act, y[o]);
                        db[f] += dz;
                        for (int c = 0; c < Ci; ++c)
                            for (int a = 0; a < k; ++a)
                                for (int bb = 0; bb < k; ++bb) {
                                    const long wi = (((long)f * Ci + c) * k + a) * k + bb;
                                    const long xi = ((long)c * mi + (u * s + a)) * mi + (v * s + bb);
                                    dw[wi] += dz * x[xi];
                                    dx[xi] += dz * w[wi];
                                }
                    }
        } else if (L[l].kind == ORC_MAXPOOL) {
            const int *am = amax + g->act_off[l + 1];
            for (int c = 0; c < Ci; ++c)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        const long o = ((long)c * mo + u) * mo + v;
                        const int a = am[o] / k, bb = am[o] % k;
                        dx[((long)c * mi + (u * s + a)) * mi + (v * s + bb)] += dy[o];
                    }
        } else {
            const double inv = 1.0 / (double)(k * k);
            for (int c = 0; c < Ci; ++c)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        const double d = dy[((long)c * mo + u) * mo + v] * inv;
                        for (int a = 0; a < k; ++a)
                            for (int bb = 0; bb < k; ++bb)
                                dx[((long)c * mi + (u * s + a)) * mi + (v * s + bb)] += d;
                    }
        }
    }
}

static void crop_patch(const double *xpad, int C0, int Hp, int Wp, int n,
                       int img, int i, int j, double *dst)
{
    for (int c = 0; c < C0; ++c)
        for (int r = 0; r < n; ++r)
            memcpy(dst + ((long)c * n + r) * n,
                   xpad + (((long)img * C0 + c) * Hp + (i + r)) * Wp + j,
                   sizeof(double) * (size_t)n);
}

/* One patch, all intermediates (for layer-by-layer checks).  patch: C0*n*n.
 * acts: orc_sizes().act_total doubles; amax: same count of ints (may be NULL);
 * pre: same count of doubles (may be NULL), see patch_forward. */
int orc_patch_forward(const orc_layer *L, int nL, int C0, int n, const double *params,
                      const double *patch, double *acts, int *amax, double *pre, int storage)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g)) return -1;
    memcpy(acts, patch, sizeof(double) * (size_t)C0 * n * n);
    if (amax) for (long t = 0; t < g.act_off[nL + 1]; ++t) amax[t] = -1;
    patch_forward(L, &g, params, acts, amax, storage, pre);
    return 0;
}

/* Forward scan.  xpad: [N][C0][Hp][Wp] (already padded); pix: [P][3] = (image,
 * i, j) in UNPADDED pixel coordinates; the patch of (i, j) is padded rows
 * i..i+n-1, columns j..j+n-1.  scores: [P][classes].  last_amax (may be NULL):
 * [P][classes] winning tap indices when the last layer is a max pool.  The net
 * must reduce the patch to 1 x 1.  storage: ORC_STORE_*.  Returns 0, or -1 on a
 * malformed net / out-of-range pixel. */
int orc_scan_forward(const orc_layer *L, int nL, int C0, int n, const double *params,
                     const double *xpad, int N, int Hp, int Wp,
                     const int *pix, long P, double *scores, int *last_amax,
                     int storage)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g) || g.m[nL] != 1) return -1;
    for (long p = 0; p < P; ++p)
        if (pix[3 * p] < 0 || pix[3 * p] >= N || pix[3 * p + 1] < 0 || pix[3 * p + 1] + n > Hp ||
            pix[3 * p + 2] < 0 || pix[3 * p + 2] + n > Wp) return -1;
    const int cls = g.C[nL];
    int fail = 0;
#pragma omp parallel
    {
        double *acts = (double *)malloc(sizeof(double) * (size_t)g.act_off[nL + 1]);
        int *amax = last_amax ? (int *)malloc(sizeof(int) * (size_t)g.act_off[nL + 1]) : NULL;
        if (!acts || (last_amax && !amax)) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long p = 0; p < P; ++p) {
            if (!acts || (last_amax && !amax)) continue;
            crop_patch(xpad, C0, Hp, Wp, n, pix[3 * p], pix[3 * p + 1], pix[3 * p + 2], acts);
            patch_forward(L, &g, params, acts, amax, storage, NULL);
            memcpy(scores + p * cls, acts + g.act_off[nL], sizeof(double) * (size_t)cls);
            if (last_amax)
                memcpy(last_amax + p * cls, amax + g.act_off[nL], sizeof(int) * (size_t)cls);
        }
        free(acts);
        free(amax);
    }
    return fail ? -2 : 0;
}

/* The same scan, keeping everything: acts [P][act_total] holds all maps of every
 * patch (map 0 = the patch itself), amax [P][act_total] the winning tap index
 * of each max-pool output (-1 elsewhere), pre [P][act_total] (may be NULL) the
 * pre-activation values of conv outputs (0 elsewhere).  By the correspondence
 * of Fig. 3, entry (u, v) of map l of the patch at (i, j) is the whole-image
 * map l at (i + D*u, j + D*v), D = product of the strides of layers 1..l. */
int orc_scan_forward_maps(const orc_layer *L, int nL, int C0, int n, const double *params,
                          const double *xpad, int N, int Hp, int Wp,
                          const int *pix, long P, double *acts, int *amax, double *pre,
                          int storage)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g)) return -1;
    for (long p = 0; p < P; ++p)
        if (pix[3 * p] < 0 || pix[3 * p] >= N || pix[3 * p + 1] < 0 || pix[3 * p + 1] + n > Hp ||
            pix[3 * p + 2] < 0 || pix[3 * p + 2] + n > Wp) return -1;
    const long na = g.act_off[nL + 1];
#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < P; ++p) {
        double *a = acts + p * na;
        int *am = amax + p * na;
        double *z = pre ? pre + p * na : NULL;
        for (long t = 0; t < na; ++t) am[t] = -1;
        if (z) memset(z, 0, sizeof(double) * (size_t)na);
        crop_patch(xpad, C0, Hp, Wp, n, pix[3 * p], pix[3 * p + 1], pix[3 * p + 2], a);
        patch_forward(L, &g, params, a, am, storage, z);
    }
    return 0;
}

/* Backward scan: each listed patch goes forward, then backward with output
 * error delta[p][classes]; parameter gradients are SUMMED over patches into
 * dparams (n_params doubles, overwritten).  dxpad (may be NULL): same shape as
 * xpad, overwritten with the scatter-add of every patch's input gradient.
 * Per-thread partial sums are combined in thread order. */
int orc_scan_backward(const orc_layer *L, int nL, int C0, int n, const double *params,
                      const double *xpad, int N, int Hp, int Wp,
                      const int *pix, long P, const double *delta,
                      double *dparams, double *dxpad, int storage)
{
    orc_geom g;
    if (geom_build(L, nL, C0, n, &g) || g.m[nL] != 1) return -1;
    for (long p = 0; p < P; ++p)
        if (pix[3 * p] < 0 || pix[3 * p] >= N || pix[3 * p + 1] < 0 || pix[3 * p + 1] + n > Hp ||
            pix[3 * p + 2] < 0 || pix[3 * p + 2] + n > Wp) return -1;
    const int cls = g.C[nL];
    const long na = g.act_off[nL + 1];
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    double *part = (double *)calloc((size_t)nthreads * (size_t)(g.n_params > 0 ? g.n_params : 1),
                                    sizeof(double));
    if (!part) return -2;
    if (dxpad) memset(dxpad, 0, sizeof(double) * (size_t)N * C0 * Hp * Wp);
    int fail = 0;
#pragma omp parallel num_threads(nthreads)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *acts = (double *)malloc(sizeof(double) * (size_t)na);
        double *grads = (double *)malloc(sizeof(double) * (size_t)na);
        int *amax = (int *)malloc(sizeof(int) * (size_t)na);
        double *mine = part + (size_t)tid * (size_t)g.n_params;
        if (!acts || !grads || !amax) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (long p = 0; p < P; ++p) {
            if (!acts || !grads || !amax) continue;
            const int img = pix[3 * p], i = pix[3 * p + 1], j = pix[3 * p + 2];
            crop_patch(xpad, C0, Hp, Wp, n, img, i, j, acts);
            patch_forward(L, &g, params, acts, amax, storage, NULL);
            memset(grads, 0, sizeof(double) * (size_t)na);
            memcpy(grads + g.act_off[nL], delta + p * cls, sizeof(double) * (size_t)cls);
            patch_backward(L, &g, params, acts, amax, grads, mine);
            if (dxpad) {
#pragma omp critical(orc_dx)
                for (int c = 0; c < C0; ++c)
                    for (int r = 0; r < n; ++r)
                        for (int q = 0; q < n; ++q)
                            dxpad[(((long)img * C0 + c) * Hp + (i + r)) * Wp + (j + q)] +=
                                grads[((long)c * n + r) * n + q];
            }
        }
        free(acts); free(grads); free(amax);
    }
    for (long t = 0; t < g.n_params; ++t) {
        double acc = 0.0;
        for (int th = 0; th < nthreads; ++th) acc += part[(size_t)th * (size_t)g.n_params + t];
        dparams[t] = acc;
    }
    free(part);
    return fail ? -2 : 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
