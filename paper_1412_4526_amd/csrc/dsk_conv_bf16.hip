// Stride-1 convolution with a d-regularly sparse kernel (paper Sec. 3.1-3.2, Algorithm 1) and its
// backward-data form (Sec. 4.1) for bf16 maps on the bf16 matrix cores: bf16 inputs and weights,
// fp32 accumulation (v_mfma_f32_32x32x16_bf16), bias and non-linearity in fp32.
//
// Same decomposition as the fp32 kernel: a workgroup owns TH=8 output rows of one residue
// class modulo d, TW=64 columns and 32 or 64 filters; the LDS tile has TH+kh-1 rows whatever d
// is.  What differs is the k index.  One matrix instruction contracts 16 values, here the 16
// channels of a chunk at one tap, and a lane supplies 8 consecutive ones.  The LDS tile is
// therefore pixel-major, [row][column][16 channels] (32 bytes per pixel), so that a lane's 8
// channels are one 16-byte read, and the weights are [tap][filter][16 channels].  The maps stay
// NCHW in HBM: the tile is transposed while it is staged.  A thread stages "items" = (pixel,
// half of the 16 channels): eight 2-byte loads, one from each channel plane, which for the
// lanes of a wave are consecutive pixels of a row (coalesced), packed into one 16-byte LDS write.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;
static constexpr int kXcds = 8;
static constexpr int TH = 8, TW = 64, CK = 16;
static constexpr int kItems = 8;        // (pixel, channel half) items per thread per chunk, at most
static constexpr int kItemsPair = 4;    // (pixel pair, channel half) items per thread per chunk, at most
static constexpr int kWq = 8;           // 16-byte pieces of the chunk's weights per thread, at most
static constexpr size_t kMaxLds = 64 * 1024;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct GbParams {
    const bf16 *in;
    void *out;
    const bf16 *wt;      // [n_fgrp][NC][taps][TF][16], zero padded
    const float *bias;   // may be null
    int N, Cin, Hin, Win, Fout, Hout, Wout;
    int kh, kw, d, off_h, off_w, act;
    int NC;              // chunks of 16 channels
    int rows, cols, n_pix;   // LDS tile: TH+kh-1 by TW+(kw-1)*d pixels; n_pix: pixels (or pixel pairs) staged per channel half
    int pp_row;          // pixel pairs per tile row (pair form)
    int n_items, n_wq;   // per thread and chunk: items, 16-byte weight pieces (LDS parts padded accordingly)
    int xs_bytes;
    int n_rowtile, n_coltile, n_fgrp;
    int nrb, full_cls;   // row blocks of d*TH rows; residue classes that have a tile in the last one (the others: nrb-1 tiles)
    long tiles, per_xcd;
};

// wt[g][ch][t][fl][cc] = w[g*TF+fl][ch*16+cc][t]                (forward)
//                      = w[ch*16+cc][g*TF+fl][taps-1-t]         (backward-data: roles swapped, taps reversed)
__global__ void __launch_bounds__(kThreads)
gb_weight_prep_kernel(const float *__restrict__ w, bf16 *__restrict__ wt, int K, int C, int taps, int NC, int TF,
                      int n_fgrp, int flip)
{
    const long total = (long)n_fgrp * NC * taps * TF * CK;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int cc = (int)(idx % CK);
    const int fl = (int)((idx / CK) % TF);
    const int t = (int)((idx / ((long)CK * TF)) % taps);
    const int ch = (int)((idx / ((long)CK * TF * taps)) % NC);
    const int g = (int)(idx / ((long)CK * TF * taps * NC));
    const int f = g * TF + fl, c = ch * CK + cc;
    float v = 0.f;
    if (!flip) {
        if (f < K && c < C) v = w[((long)f * C + c) * taps + t];
    } else {
        if (f < C && c < K) v = w[((long)c * C + f) * taps + (taps - 1 - t)];
    }
    wt[idx] = f32_to_bf16(v);
}

// PAIR (maps with an even number of columns): an item is (pixel PAIR, channel half).  Every row of
// a plane then starts at an even element, so two neighbouring pixels starting at an even column
// are one aligned 4-byte load: half as many loads and staging registers, and the two pixels are
// separated when they are packed for LDS.
template <typename TO, int WM, bool PAIR>
__global__ void __launch_bounds__(kThreads, 2)
gemm_conv_bf16_kernel(GbParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int TF = WM * 32, NI = PAIR ? kItemsPair : kItems;
    unsigned char *xs = smem;                  // [rows*cols pixels][16 channels] bf16
    unsigned char *wsm = smem + p.xs_bytes;    // [taps][TF][16 channels] bf16

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lo = lane & 31, hi = lane >> 5;

    // XCD-aware tile order: neighbouring tiles share one XCD's L2
    long tile = (long)(blockIdx.x % kXcds) * p.per_xcd + blockIdx.x / kXcds;
    if (tile >= p.tiles) return;
    const int fg = (int)(tile % p.n_fgrp); tile /= p.n_fgrp;
    const int ct = (int)(tile % p.n_coltile); tile /= p.n_coltile;
    const int rt = (int)(tile % p.n_rowtile);
    const int n = (int)(tile / p.n_rowtile);
    // row tiles are numbered class by class, down the map within a class: tiles that follow each other
    // (one XCD, the same time) share input rows; different residue classes share none
    const int nf = p.full_cls * p.nrb;
    int cls, rb;
    if (rt < nf) {
        cls = rt / p.nrb; rb = rt - cls * p.nrb;
    } else {
        const int q = (rt - nf) / (p.nrb - 1);
        cls = p.full_cls + q; rb = rt - nf - q * (p.nrb - 1);
    }
    const int u0 = rb * p.d * TH + cls;
    const int v0 = ct * TW;

    const unsigned HW = (unsigned)(p.Hin * p.Win);
    const int taps = p.kh * p.kw;
    const bf16 *in_n = p.in + (long)n * p.Cin * (long)HW;
    const BufRsrc rx = buf_rsrc(in_n, p.in + (long)p.N * p.Cin * (long)HW);

    // Item it = tid + 256*i: channel half g = it / n_pix, pixel it % n_pix of the tile.  voff[i] is
    // where channel 8*g of the chunk is read for that pixel, relative to the chunk's first
    // channel; pixels outside the map (and the padding of the item list) read offset 0, which
    // is a valid address, and bit i of `zero` turns them into zeros at the LDS write.
    // PAIR: n_pix counts pixel pairs (pp_row per tile row); pair jp of a row is tile columns
    // 2*jp - par and 2*jp + 1 - par, where par makes the first one an even map column; lpix[i] is
    // the LDS pixel index of the first (the second follows it) and bits 8+i / 16+i of `zero`
    // say that the first / second column lies outside the tile and is not written.
    unsigned voff[NI];
    int lpix[PAIR ? NI : 1];
    unsigned zero = 0;
    const int par = PAIR ? (v0 - p.off_w) & 1 : 0;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int it = tid + i * kThreads;
        const int g = it >= p.n_pix ? 1 : 0, pi = it - g * p.n_pix;
        if (PAIR) {
            const int r = pi / p.pp_row, c = 2 * (pi - r * p.pp_row) - par;
            const int irow = u0 + r * p.d - p.off_h, icol = v0 + c - p.off_w;      // icol is even
            const bool ok = it < 2 * p.n_pix && irow >= 0 && irow < p.Hin && icol >= 0 && icol < p.Win;
            voff[i] = ok ? (unsigned)(8 * g) * HW + (unsigned)(irow * p.Win + icol) : 0u;
            lpix[i] = r * p.cols + c;
            zero |= ok ? 0u : 1u << i;
            zero |= it < 2 * p.n_pix && c >= 0 && c < p.cols ? 0u : 1u << (8 + i);
            zero |= it < 2 * p.n_pix && c + 1 >= 0 && c + 1 < p.cols ? 0u : 1u << (16 + i);
        } else {
            const int r = pi / p.cols, c = pi - r * p.cols;
            const int irow = u0 + r * p.d - p.off_h, icol = v0 + c - p.off_w;
            const bool ok = it < 2 * p.n_pix && irow >= 0 && irow < p.Hin && icol >= 0 && icol < p.Win;
            voff[i] = ok ? (unsigned)(8 * g) * HW + (unsigned)(irow * p.Win + icol) : 0u;
            zero |= ok ? 0u : 1u << i;
        }
    }

    f32x16 acc[WM][4];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
        for (int wn = 0; wn < 4; ++wn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[wm][wn][i] = 0.f;

    unsigned xr[NI][8];      // one 2-byte value each (PAIR: two, of neighbouring pixels)
    u32x4 wv[kWq];
    // Every load is issued unconditionally: a load under a condition would be waited for on the spot.
    auto fetch = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * CK;
        if (c0 + CK <= p.Cin) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    xr[i][j] = PAIR ? __builtin_amdgcn_raw_buffer_load_b32(rx, (int)(voff[i] * 2u), (int)((unsigned)(c0 + j) * HW * 2u), 0)
                                    : __builtin_amdgcn_raw_buffer_load_b16(rx, (int)(voff[i] * 2u), (int)((unsigned)(c0 + j) * HW * 2u), 0);
        } else {
            // last chunk of a padded channel count: channels at or beyond Cin meet zero weights;
            // the chunk's first channel is read instead so that the address stays inside the tensor
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int g8 = tid + i * kThreads >= p.n_pix ? 8 : 0;
                const unsigned pix = voff[i] - (unsigned)g8 * HW * ((zero >> i) & 1u ? 0u : 1u);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const unsigned off = c0 + g8 + j < p.Cin ? voff[i] + (unsigned)j * HW : pix;
                    xr[i][j] = PAIR ? __builtin_amdgcn_raw_buffer_load_b32(rx, (int)(off * 2u), (int)((unsigned)c0 * HW * 2u), 0)
                                    : __builtin_amdgcn_raw_buffer_load_b16(rx, (int)(off * 2u), (int)((unsigned)c0 * HW * 2u), 0);
                }
            }
        }
        const bf16 *wsrc = p.wt + ((long)fg * p.NC + ch) * taps * TF * CK;
        const BufRsrc rw = buf_rsrc(wsrc, wsrc + (long)taps * TF * CK);      // the padding of the LDS part reads zero
#pragma unroll
        for (int q = 0; q < kWq; ++q)
            wv[q] = __builtin_amdgcn_raw_buffer_load_b128(rw, (q * kThreads + tid) * 16, 0, 0);
    };

    // per-lane LDS byte addresses: B = pixel (row 2*wave, column lo) + 16 bytes for lanes 32..63
    // (channels 8..15), A = filter lo likewise
    const unsigned char *xlane = xs + ((2 * wave) * p.cols + lo) * 32 + hi * 16;
    const unsigned char *wlane = wsm + lo * 32 + hi * 16;

    fetch(0);
    for (int ch = 0; ch < p.NC; ++ch) {
        __syncthreads();      // every wave is done reading the previous chunk
        // The loaded halves are packed here, not where they were fetched: packed early (which the
        // compiler would do to halve the registers they occupy) every pair of loads is waited for
        // on the spot, and a chunk then costs 32 memory round trips instead of one.
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(xr[i][j]));
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (i < p.n_items) {
                const int it = tid + i * kThreads;
                const int g = it >= p.n_pix ? 1 : 0;
                const bool z = (zero >> i) & 1u;
                if (PAIR) {
                    u32x4 va, vb;      // the low halves belong to the first pixel, the high halves to the second
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const unsigned q0 = xr[i][2 * j], q1 = xr[i][2 * j + 1];
                        va[j] = z ? 0u : (q0 & 0xffffu) | (q1 << 16);
                        vb[j] = z ? 0u : (q0 >> 16) | (q1 & 0xffff0000u);
                    }
                    if (!((zero >> (8 + i)) & 1u)) *(u32x4 *)(xs + lpix[i] * 32 + g * 16) = va;
                    if (!((zero >> (16 + i)) & 1u)) *(u32x4 *)(xs + (lpix[i] + 1) * 32 + g * 16) = vb;
                } else {
                    u32x4 v;
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = z ? 0u : xr[i][2 * j] | (xr[i][2 * j + 1] << 16);
                    if (it < 2 * p.n_pix) *(u32x4 *)(xs + (it - g * p.n_pix) * 32 + g * 16) = v;
                }
            }
#pragma unroll
        for (int q = 0; q < kWq; ++q)
            if (q < p.n_wq) ((u32x4 *)wsm)[q * kThreads + tid] = wv[q];
        __syncthreads();
        fetch(ch + 1 < p.NC ? ch + 1 : ch);      // in flight while the matrix cores run (the last one is not used)

        // ---- matrix cores: one instruction per tap and accumulator tile, k = the chunk's 16 channels
        for (int ta = 0; ta < p.kh; ++ta) {
            for (int tb = 0; tb < p.kw; ++tb) {
                const int xo = (ta * p.cols + tb * p.d) * 32, wo = (ta * p.kw + tb) * TF * 32;
                bf16x8 A[WM], B[4];
#pragma unroll
                for (int wm = 0; wm < WM; ++wm) A[wm] = *(const bf16x8 *)(wlane + wo + wm * 32 * 32);
#pragma unroll
                for (int wn = 0; wn < 4; ++wn)
                    B[wn] = *(const bf16x8 *)(xlane + xo + ((wn >> 1) * p.cols + (wn & 1) * 32) * 32);
#pragma unroll
                for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                    for (int wn = 0; wn < 4; ++wn)
                        acc[wm][wn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[wm], B[wn], acc[wm][wn], 0, 0, 0);
            }
        }
    }

    // ---- bias, non-linearity, store (register i of a lane: filter 8*(i/4) + i%4 + 4*hi of its block)
    const long plane = (long)p.Hout * p.Wout;
    TO *out_n = (TO *)p.out + ((long)n * p.Fout + (long)fg * TF) * plane;
    const int f_left = p.Fout - fg * TF;
    // The biases of this lane's filters, fetched together BEFORE the first store: loaded where they
    // are used, each load is waited for on the spot (it may not pass the stores before it), one
    // memory round trip per output.  Filters beyond Fout read zero through the descriptor's range.
    float bv[WM][16];
    {
        const BufRsrc rb = buf_rsrc(p.bias, p.bias + (p.bias ? p.Fout : 0));
#pragma unroll
        for (int wm = 0; wm < WM; ++wm)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                bv[wm][i] = buf_ld(rb, p.bias, (unsigned)(fg * TF + wm * 32 + 8 * (i / 4) + (i % 4) + 4 * hi), 0u);
#pragma unroll
        for (int wm = 0; wm < WM; ++wm)
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(bv[wm][i]));
    }
#pragma unroll
    for (int wn = 0; wn < 4; ++wn) {
        const int row = u0 + (2 * wave + (wn >> 1)) * p.d;
        const int col = v0 + (wn & 1) * 32 + lo;
        if (row >= p.Hout || col >= p.Wout) continue;
        TO *o = out_n + (long)row * p.Wout + col + (hi ? 4 * plane : 0);
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int fl = wm * 32 + 8 * (i / 4) + (i % 4);
                if (fl + 4 * hi < f_left) stf(o, (long)fl * plane, act_apply(p.act, acc[wm][wn][i] + bv[wm][i]));
            }
        }
    }
}

struct GbPlan {
    bool ok;
    int WM, TF, NC, rows, cols, n_pix, pp_row, n_items, n_wq, xs_bytes, n_fgrp, n_rowtile, n_coltile, nrb, full_cls;
    bool pair;
    long tiles;
    size_t lds_bytes, wt_bytes;
};

// Cin / Fout: channel and output counts of the GEMM (swapped for backward-data)
static GbPlan gb_plan(int N, int Cin, int Win, int Fout, int Hout, int Wout, int kh, int kw, int d)
{
    GbPlan g{};
    if (Cin < CK) return g;        // a first layer with 3 channels would be 13/16 padding
    g.rows = TH + kh - 1;
    const long cols = (long)TW + (long)(kw - 1) * d;
    const long taps = (long)kh * kw;
    if (cols > 4096 || taps > 1024) return g;
    g.cols = (int)cols;
    g.pair = Win % 2 == 0;
    g.pp_row = g.cols / 2 + 1;
    g.n_pix = g.pair ? g.rows * g.pp_row : g.rows * g.cols;
    g.n_items = (2 * g.n_pix + kThreads - 1) / kThreads;
    if (g.pair && g.n_items > kItemsPair) {      // too many pairs for the registers set aside: single pixels
        g.pair = false;
        g.n_pix = g.rows * g.cols;
        g.n_items = (2 * g.n_pix + kThreads - 1) / kThreads;
    }
    if (g.n_items > kItems) return g;
    g.xs_bytes = (g.rows * g.cols * 32 + 255) & ~255;
    for (int wm = 2; wm >= 1; --wm) {
        if (wm == 2 && Fout <= 32) continue;
        const long wbytes = taps * wm * 32 * CK * 2;
        const int n_wq = (int)((wbytes + 16 * kThreads - 1) / (16 * kThreads));
        if (n_wq > kWq || (size_t)g.xs_bytes + (size_t)n_wq * kThreads * 16 > kMaxLds) continue;
        g.WM = wm;
        g.n_wq = n_wq;
        break;
    }
    if (g.WM == 0) return g;
    g.TF = g.WM * 32;
    g.lds_bytes = (size_t)g.xs_bytes + (size_t)g.n_wq * kThreads * 16;
    g.n_fgrp = (Fout + g.TF - 1) / g.TF;
    g.NC = (Cin + CK - 1) / CK;
    g.wt_bytes = (2 * (size_t)g.n_fgrp * g.NC * taps * g.TF * CK + 255) & ~(size_t)255;
    {
        const int nrb = (Hout + d * TH - 1) / (d * TH);
        const int last = Hout - (nrb - 1) * d * TH;
        g.n_rowtile = (nrb - 1) * d + (last < d ? last : d);
        g.nrb = nrb;
        g.full_cls = last < d ? last : d;
    }
    g.n_coltile = (Wout + TW - 1) / TW;
    g.tiles = (long)N * g.n_rowtile * g.n_coltile * g.n_fgrp;
    g.ok = true;
    return g;
}

static int gb_run(const void *in, void *out, const float *w, const float *bias, int N, int Cin, int Hin, int Win,
                  int Fout, int Hout, int Wout, int kh, int kw, int d, int off, int act, int flip, int K, int C,
                  dsk_dtype tout, void *ws, hipStream_t st)
{
    const GbPlan g = gb_plan(N, Cin, Win, Fout, Hout, Wout, kh, kw, d);
    if (!g.ok) return DSK_ESHAPE;
    const int taps = kh * kw;
    bf16 *wt = (bf16 *)ws;
    {
        const long total = (long)g.n_fgrp * g.NC * taps * g.TF * CK;
        gb_weight_prep_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
            w, wt, K, C, taps, g.NC, g.TF, g.n_fgrp, flip);
    }
    GbParams p{};
    p.in = (const bf16 *)in; p.out = out; p.wt = wt; p.bias = bias;
    p.N = N; p.Cin = Cin; p.Hin = Hin; p.Win = Win; p.Fout = Fout; p.Hout = Hout; p.Wout = Wout;
    p.kh = kh; p.kw = kw; p.d = d; p.off_h = off ? (kh - 1) * d : 0; p.off_w = off ? (kw - 1) * d : 0;
    p.act = act;
    p.NC = g.NC; p.rows = g.rows; p.cols = g.cols; p.n_pix = g.n_pix; p.pp_row = g.pp_row; p.n_items = g.n_items;
    p.n_wq = g.n_wq;
    p.xs_bytes = g.xs_bytes;
    p.n_rowtile = g.n_rowtile; p.n_coltile = g.n_coltile; p.n_fgrp = g.n_fgrp; p.nrb = g.nrb; p.full_cls = g.full_cls;
    p.tiles = g.tiles;
    p.per_xcd = (g.tiles + kXcds - 1) / kXcds;
    if (p.per_xcd * kXcds > 0x7fffffffL) return DSK_ESHAPE;
    const unsigned grid = (unsigned)(p.per_xcd * kXcds);
#define DSK_GB_LAUNCH(TO, WM, PAIR) gemm_conv_bf16_kernel<TO, WM, PAIR><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p)
    if (tout == DSK_BF16) {
        if (g.WM == 2 && g.pair) DSK_GB_LAUNCH(bf16, 2, true);
        else if (g.WM == 2) DSK_GB_LAUNCH(bf16, 2, false);
        else if (g.pair) DSK_GB_LAUNCH(bf16, 1, true);
        else DSK_GB_LAUNCH(bf16, 1, false);
    } else {
        if (g.WM == 2 && g.pair) DSK_GB_LAUNCH(float, 2, true);
        else if (g.WM == 2) DSK_GB_LAUNCH(float, 2, false);
        else if (g.pair) DSK_GB_LAUNCH(float, 1, true);
        else DSK_GB_LAUNCH(float, 1, false);
    }
#undef DSK_GB_LAUNCH
    return check_launch();
}

// ---- entry points for the dispatcher (bf16 input maps only)
size_t conv_bf16_ws_bytes(int which, const ConvShape &s)
{
    const GbPlan g = which == DSK_WS_CONV_FWD ? gb_plan(s.N, s.C, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d)
                                              : gb_plan(s.N, s.K, s.Wo, s.C, s.H, s.W, s.kh, s.kw, s.d);
    return g.ok ? g.wt_bytes : 0;
}

bool conv_bf16_supported(int which, const ConvShape &s)
{
    if ((long)s.H * s.W >= (1L << 28) || (long)s.C * s.H * s.W >= (1L << 30) ||
        (long)s.K * s.Ho * s.Wo >= (1L << 30))
        return false;
    if (s.kh == 1 && s.kw == 1) return false;      // 1x1 layers have their own kernel
    if (which == DSK_WS_CONV_FWD) return gb_plan(s.N, s.C, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d).ok;
    if (which == DSK_WS_CONV_BWD_DATA) return gb_plan(s.N, s.K, s.Wo, s.C, s.H, s.W, s.kh, s.kw, s.d).ok;
    return false;
}

int launch_conv_fwd_bf16(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                         dsk_dtype out, int act, void *ws, hipStream_t st)
{
    return gb_run(x, y, w, b, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d, 0, act, 0, s.K, s.C, out, ws, st);
}

int launch_conv_bwd_data_bf16(const void *dy, const float *w, void *dx, const ConvShape &s, dsk_dtype out, void *ws,
                              hipStream_t st)
{
    return gb_run(dy, dx, w, nullptr, s.N, s.K, s.Ho, s.Wo, s.C, s.H, s.W, s.kh, s.kw, s.d, 1, DSK_ACT_NONE, 1,
                  s.K, s.C, out, ws, st);
}

} // namespace dsk
