/*
 * TEST INFRASTRUCTURE -- the CPU oracle for video (3-D) networks.  Not part of
 * the product: only the tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.
 *
 * Literal cube-by-cube scanning: the paper's closing section proposes carrying
 * its method over to video with 3-D convolution and 3-D pooling, where the
 * baseline is a classifier that looks at one nt x n x n cube per labelled
 * voxel.  For every requested voxel the cube is cropped from the padded video
 * and pushed through the ORIGINAL strided 3-D CNN; backward feeds each cube's
 * output error through the textbook backward pass and sums the per-cube
 * parameter gradients (the 3-D counterpart of Sec. 1.1, Fig. 1(a), Sec. 4.3).
 *
 * Nothing here knows about dilation / sparse kernels.  fp64, plain loops.
 *
 * Maps are [C][T][H][W]; a layer has a temporal kernel size kt and stride st
 * and a square spatial kernel k with stride s ("valid", floor):
 *   conv    y[f][q][u][v] = act(b[f] + sum_{c,e,a,b} w[f][c][e][a][b]
 *                                   x[c][q*st+e][u*s+a][v*s+b])      (cross-correlation)
 *   maxpool y[c][q][u][v] = max over the kt*k*k taps; the winning tap's index
 *           (e*k + a)*k + b is recorded; taps are scanned in that order and
 *           replaced only on strict '>', so the lowest index wins ties
 *   avgpool mean of the kt*k*k taps
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
    int k;    /* spatial kernel size (square) */
    int s;    /* spatial stride */
    int kt;   /* temporal kernel size */
    int st;   /* temporal stride */
    int act;  /* conv: ORC_ACT_* */
} orc3_layer;

#define ORC3_MAX_LAYERS 64

typedef struct {
    int nL;
    int C[ORC3_MAX_LAYERS + 1];  /* channels of map l (map 0 = the cube) */
    int m[ORC3_MAX_LAYERS + 1];  /* spatial size of map l */
    int mt[ORC3_MAX_LAYERS + 1]; /* temporal size of map l */
    long act_off[ORC3_MAX_LAYERS + 2];
    long par_off[ORC3_MAX_LAYERS + 1];
    long n_params;
} orc3_geom;

static long map_size(const orc3_geom *g, int l)
{
    return (long)g->C[l] * g->mt[l] * g->m[l] * g->m[l];
}

static int geom_build(const orc3_layer *L, int nL, int C0, int nt, int n, orc3_geom *g)
{
    if (nL < 1 || nL > ORC3_MAX_LAYERS || C0 < 1 || n < 1 || nt < 1) return -1;
    g->nL = nL;
    g->C[0] = C0; g->m[0] = n; g->mt[0] = nt;
    g->act_off[0] = 0;
    long po = 0;
    for (int l = 0; l < nL; ++l) {
        if (L[l].k < 1 || L[l].s < 1 || L[l].k > g->m[l]) return -1;
        if (L[l].kt < 1 || L[l].st < 1 || L[l].kt > g->mt[l]) return -1;
        g->m[l + 1] = (g->m[l] - L[l].k) / L[l].s + 1;
        g->mt[l + 1] = (g->mt[l] - L[l].kt) / L[l].st + 1;
        g->act_off[l + 1] = g->act_off[l] + map_size(g, l);
        g->par_off[l] = po;
        if (L[l].kind == ORC_CONV) {
            if (L[l].K < 1) return -1;
            g->C[l + 1] = L[l].K;
            po += (long)L[l].K * g->C[l] * L[l].kt * L[l].k * L[l].k + L[l].K;
        } else if (L[l].kind == ORC_MAXPOOL || L[l].kind == ORC_AVGPOOL) {
            g->C[l + 1] = g->C[l];
        } else {
            return -1;
        }
    }
    g->act_off[nL + 1] = g->act_off[nL] + map_size(g, nL);
    g->n_params = po;
    return 0;
}

/* C[l], mt[l], m[l], act_off[l] for l = 0..nL (act_off has nL+2 entries: the
 * last is the total), par_off[l] for l < nL; *n_params the parameter count. */
int orc3_geometry(const orc3_layer *L, int nL, int C0, int nt, int n,
                  int *C, int *mt, int *m, long *act_off, long *par_off, long *n_params)
{
    orc3_geom g;
    if (geom_build(L, nL, C0, nt, n, &g)) return -1;
    for (int l = 0; l <= nL; ++l) { C[l] = g.C[l]; mt[l] = g.mt[l]; m[l] = g.m[l]; act_off[l] = g.act_off[l]; }
    act_off[nL + 1] = g.act_off[nL + 1];
    for (int l = 0; l < nL; ++l) par_off[l] = g.par_off[l];
    *n_params = g.n_params;
    return 0;
}

static double act_apply(int act, double z)
{
    if (act == ORC_ACT_RELU) return z > 0.0 ? z : 0.0;
    if (act == ORC_ACT_TANH) return tanh(z);
    return z;
}

static double act_grad_from_output(int act, double y)
{
    if (act == ORC_ACT_RELU) return y > 0.0 ? 1.0 : 0.0;
    if (act == ORC_ACT_TANH) return 1.0 - y * y;
    return 1.0;
}

/* index of x[c][t][r][q] in a [C][mt][m][m] map */
#define AT(c, t, r, q, mt, m) ((((long)(c) * (mt) + (t)) * (m) + (r)) * (m) + (q))

/* Forward of the original CNN on one cube (already at acts[0...]); fills every
 * later map; amax gets the winning tap of each max-pool output at the offsets
 * of that map (other entries untouched). */
static void cube_forward(const orc3_layer *L, const orc3_geom *g, const double *params,
                         double *acts, int *amax)
{
    for (int l = 0; l < g->nL; ++l) {
        const int Ci = g->C[l], mi = g->m[l], ti = g->mt[l];
        const int Co = g->C[l + 1], mo = g->m[l + 1], to = g->mt[l + 1];
        const int k = L[l].k, s = L[l].s, kt = L[l].kt, st = L[l].st;
        const double *x = acts + g->act_off[l];
        double *y = acts + g->act_off[l + 1];
        int *am = amax ? amax + g->act_off[l + 1] : NULL;
        for (int f = 0; f < Co; ++f)
            for (int q = 0; q < to; ++q)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        const long o = AT(f, q, u, v, to, mo);
                        if (L[l].kind == ORC_CONV) {
                            const double *w = params + g->par_off[l];
                            const double *b = w + (long)Co * Ci * kt * k * k;
                            double acc = b[f];
                            for (int c = 0; c < Ci; ++c)
                                for (int e = 0; e < kt; ++e)
                                    for (int a = 0; a < k; ++a)
                                        for (int bb = 0; bb < k; ++bb)
                                            acc += w[((((long)f * Ci + c) * kt + e) * k + a) * k + bb] *
                                                   x[AT(c, q * st + e, u * s + a, v * s + bb, ti, mi)];
                            y[o] = act_apply(L[l].act, acc);
                        } else if (L[l].kind == ORC_MAXPOOL) {
                            double best = x[AT(f, q * st, u * s, v * s, ti, mi)];
                            int bi = 0;
                            for (int e = 0; e < kt; ++e)
                                for (int a = 0; a < k; ++a)
                                    for (int bb = 0; bb < k; ++bb) {
                                        const double t = x[AT(f, q * st + e, u * s + a, v * s + bb, ti, mi)];
                                        if (t > best) { best = t; bi = (e * k + a) * k + bb; }
                                    }
                            y[o] = best;
                            if (am) am[o] = bi;
                        } else {
                            double acc = 0.0;
                            for (int e = 0; e < kt; ++e)
                                for (int a = 0; a < k; ++a)
                                    for (int bb = 0; bb < k; ++bb)
                                        acc += x[AT(f, q * st + e, u * s + a, v * s + bb, ti, mi)];
                            y[o] = acc / (double)(kt * k * k);
                        }
                    }
    }
}

/* Textbook backward on one cube.  grads: dLoss/dmap at each map's offsets; the
 * last map's entry is the caller's, all earlier ones must be zero on entry.
 * dparams is accumulated. */
static void cube_backward(const orc3_layer *L, const orc3_geom *g, const double *params,
                          const double *acts, const int *amax, double *grads, double *dparams)
{
    for (int l = g->nL - 1; l >= 0; --l) {
        const int Ci = g->C[l], mi = g->m[l], ti = g->mt[l];
        const int Co = g->C[l + 1], mo = g->m[l + 1], to = g->mt[l + 1];
        const int k = L[l].k, s = L[l].s, kt = L[l].kt, st = L[l].st;
        const double *x = acts + g->act_off[l];
        const double *y = acts + g->act_off[l + 1];
        const double *dy = grads + g->act_off[l + 1];
        double *dx = grads + g->act_off[l];
        for (int f = 0; f < Co; ++f)
            for (int q = 0; q < to; ++q)
                for (int u = 0; u < mo; ++u)
                    for (int v = 0; v < mo; ++v) {
                        const long o = AT(f, q, u, v, to, mo);
                        if (L[l].kind == ORC_CONV) {
                            const double *w = params + g->par_off[l];
                            double *dw = dparams + g->par_off[l];
                            double *db = dw + (long)Co * Ci * kt * k * k;
                            const double dz = dy[o] * act_grad_from_output(L[l].act, y[o]);
                            db[f] += dz;
                            for (int c = 0; c < Ci; ++c)
                                for (int e = 0; e < kt; ++e)
                                    for (int a = 0; a < k; ++a)
                                        for (int bb = 0; bb < k; ++bb) {
                                            const long wi = ((((long)f * Ci + c) * kt + e) * k + a) * k + bb;
                                            const long xi = AT(c, q * st + e, u * s + a, v * s + bb, ti, mi);
                                            dw[wi] += dz * x[xi];
                                            dx[xi] += dz * w[wi];
                                        }
                        } else if (L[l].kind == ORC_MAXPOOL) {
                            const int idx = amax[g->act_off[l + 1] + o];
                            const int e = idx / (k * k), a = (idx / k) % k, bb = idx % k;
                            dx[AT(f, q * st + e, u * s + a, v * s + bb, ti, mi)] += dy[o];
                        } else {
                            const double d = dy[o] / (double)(kt * k * k);
                            for (int e = 0; e < kt; ++e)
                                for (int a = 0; a < k; ++a)
                                    for (int bb = 0; bb < k; ++bb)
                                        dx[AT(f, q * st + e, u * s + a, v * s + bb, ti, mi)] += d;
                        }
                    }
    }
}

/* xpad: [N][C0][Tp][Hp][Wp]; the cube of voxel (img, t, i, j) is padded frames
 * t..t+nt-1, rows i..i+n-1, columns j..j+n-1 */
static void crop_cube(const double *xpad, int C0, int Tp, int Hp, int Wp, int nt, int n,
                      const int *vox, double *dst)
{
    for (int c = 0; c < C0; ++c)
        for (int e = 0; e < nt; ++e)
            for (int r = 0; r < n; ++r)
                memcpy(dst + AT(c, e, r, 0, nt, n),
                       xpad + ((((long)vox[0] * C0 + c) * Tp + (vox[1] + e)) * Hp + (vox[2] + r)) * Wp + vox[3],
                       sizeof(double) * (size_t)n);
}

static int vox_ok(const int *vox, long P, int N, int Tp, int Hp, int Wp, int nt, int n)
{
    for (long p = 0; p < P; ++p) {
        const int *v = vox + 4 * p;
        if (v[0] < 0 || v[0] >= N || v[1] < 0 || v[1] + nt > Tp || v[2] < 0 || v[2] + n > Hp ||
            v[3] < 0 || v[3] + n > Wp) return 0;
    }
    return 1;
}

/* Forward scan keeping everything.  vox: [P][4] = (video, t, i, j) in UNPADDED
 * coordinates.  acts [P][act_total]: all maps of every cube (map 0 = the cube);
 * amax [P][act_total] (may be NULL): winning taps of max-pool outputs, -1
 * elsewhere.  Entry (q, u, v) of map l of the cube at (t, i, j) is the whole-video
 * map l at (t + Dt*q, i + D*u, j + D*v), Dt / D = products of the temporal /
 * spatial strides of layers 1..l (the 3-D form of Fig. 3's correspondence). */
int orc3_scan_forward_maps(const orc3_layer *L, int nL, int C0, int nt, int n, const double *params,
                           const double *xpad, int N, int Tp, int Hp, int Wp,
                           const int *vox, long P, double *acts, int *amax)
{
    orc3_geom g;
    if (geom_build(L, nL, C0, nt, n, &g)) return -1;
    if (!vox_ok(vox, P, N, Tp, Hp, Wp, nt, n)) return -1;
    const long na = g.act_off[nL + 1];
#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < P; ++p) {
        double *a = acts + p * na;
        int *am = amax ? amax + p * na : NULL;
        if (am) for (long t = 0; t < na; ++t) am[t] = -1;
        crop_cube(xpad, C0, Tp, Hp, Wp, nt, n, vox + 4 * p, a);
        cube_forward(L, &g, params, a, am);
    }
    return 0;
}

/* Scores only: scores [P][classes]; the net must reduce the cube to 1x1x1. */
int orc3_scan_forward(const orc3_layer *L, int nL, int C0, int nt, int n, const double *params,
                      const double *xpad, int N, int Tp, int Hp, int Wp,
                      const int *vox, long P, double *scores)
{
    orc3_geom g;
    if (geom_build(L, nL, C0, nt, n, &g) || g.m[nL] != 1 || g.mt[nL] != 1) return -1;
    if (!vox_ok(vox, P, N, Tp, Hp, Wp, nt, n)) return -1;
    const long na = g.act_off[nL + 1];
    const int cls = g.C[nL];
    int fail = 0;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)na);
        if (!a) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long p = 0; p < P; ++p) {
            if (!a) continue;
            crop_cube(xpad, C0, Tp, Hp, Wp, nt, n, vox + 4 * p, a);
            cube_forward(L, &g, params, a, NULL);
            memcpy(scores + p * cls, a + g.act_off[nL], sizeof(double) * (size_t)cls);
        }
        free(a);
    }
    return fail ? -2 : 0;
}

/* Backward scan: each listed cube goes forward, then backward with output error
 * delta[p][classes]; parameter gradients are SUMMED over cubes into dparams
 * (overwritten).  dxpad (may be NULL): same shape as xpad, overwritten with the
 * scatter-add of every cube's input gradient.  Per-thread partial sums are
 * combined in thread order. */
int orc3_scan_backward(const orc3_layer *L, int nL, int C0, int nt, int n, const double *params,
                       const double *xpad, int N, int Tp, int Hp, int Wp,
                       const int *vox, long P, const double *delta,
                       double *dparams, double *dxpad)
{
    orc3_geom g;
    if (geom_build(L, nL, C0, nt, n, &g) || g.m[nL] != 1 || g.mt[nL] != 1) return -1;
    if (!vox_ok(vox, P, N, Tp, Hp, Wp, nt, n)) return -1;
    const int cls = g.C[nL];
    const long na = g.act_off[nL + 1];
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    double *part = (double *)calloc((size_t)nthreads * (size_t)(g.n_params > 0 ? g.n_params : 1), sizeof(double));
    if (!part) return -2;
    if (dxpad) memset(dxpad, 0, sizeof(double) * (size_t)N * C0 * Tp * Hp * Wp);
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
            const int *v = vox + 4 * p;
            crop_cube(xpad, C0, Tp, Hp, Wp, nt, n, v, acts);
            cube_forward(L, &g, params, acts, amax);
            memset(grads, 0, sizeof(double) * (size_t)na);
            memcpy(grads + g.act_off[nL], delta + p * cls, sizeof(double) * (size_t)cls);
            cube_backward(L, &g, params, acts, amax, grads, mine);
            if (dxpad) {
#pragma omp critical(orc3_dx)
                for (int c = 0; c < C0; ++c)
                    for (int e = 0; e < nt; ++e)
                        for (int r = 0; r < n; ++r)
                            for (int q = 0; q < n; ++q)
                                dxpad[((((long)v[0] * C0 + c) * Tp + (v[1] + e)) * Hp + (v[2] + r)) * Wp + (v[3] + q)] +=
                                    grads[AT(c, e, r, q, nt, n)];
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
