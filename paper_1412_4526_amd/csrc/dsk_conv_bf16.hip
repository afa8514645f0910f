// Stride-1 convolution with a d-regularly sparse kernel (paper Sec. 3.1-3.2, Algorithm 1) and its
// backward-data form (Sec. 4.1) for bf16 maps on the bf16 matrix cores: bf16 inputs and weights,
// fp32 accumulation (v_mfma_f32_32x32x16_bf16), bias and non-linearity in fp32.
//
// Same decomposition as the fp32 kernel: a workgroup owns TH=8 output rows of one residue
// class modulo d, TW=64 columns and 32 or 64 filters; the LDS tile has TH+kh-1 rows whatever d
// is.  What differs is the k index.  One matrix instruction contracts 16 values, here the 16
// channels of a chunk at one tap, and a lane supplies 8 consecutive ones (16 bytes).  The LDS
// tile is therefore [channel half][row][column][8 channels] and the weights are
// [tap][channel half][filter][8 channels]: the 32 lanes of a half-wave read 32 consecutive
// 16-byte pieces (no bank conflicts).  The maps stay NCHW in HBM: the tile is transposed while
// it is staged.  A thread stages "items" = (four neighbouring pixels, half of the 16 channels):
// eight 8-byte loads, one from each channel plane, turned into four 16-byte LDS writes (one per
// pixel) by sixteen byte permutes.
//
// A wave owns FOUR rows of the tile and one 32-column block.  Tap row ta of tile row j reads LDS
// row j+ta, so the operands of LDS row r serve every (j, ta) with j+ta = r: kh+3 operand reads
// per tap column feed 4*kh matrix instructions per 32 filters.
#include "dsk_internal.h"

namespace dsk {

static constexpr int kThreads = 256;
static constexpr int kXcds = 8;
static constexpr int TH = 8, TW = 64, CK = 16;
static constexpr int kItems = 8;        // (pixel, channel half) items per thread per chunk, at most
static constexpr int kWq = 8;           // 16-byte pieces of the chunk's weights per thread, at most
static constexpr size_t kMaxLds = 64 * 1024;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

struct GbParams {
    const bf16 *in;
    void *out;
    const bf16 *wt;      // [n_fgrp][NC][taps][2][TF][8], zero padded
    const float *bias;   // may be null
    int N, Cin, Hin, Win, Fout, Hout, Wout;
    int kh, kw, d, off_h, off_w, act;
    int zero_fill;       // pixels outside the map count as zeros (backward-data); else they only feed outputs that are not stored
    int NC;              // chunks of 16 channels
    int rows, cols;      // tile: TH+kh-1 rows by TW+(kw-1)*d columns
    int cols_p;          // LDS row pitch in pixels
    int gpr;             // groups of four pixels per tile row (quad form)
    int n_pix;           // items per channel half: pixels, or groups of four
    int n_items, n_wq;   // per thread and chunk: items, 16-byte weight pieces (LDS parts padded accordingly)
    int xs_bytes;
    int n_rowtile, n_coltile, n_fgrp;
    int nrb, full_cls;   // row blocks of d*TH rows; residue classes that have a tile in the last one (the others: nrb-1 tiles)
    long tiles, per_xcd;
};

// wt[g][ch][t][h][fl][cc] = w[g*TF+fl][ch*16+8*h+cc][t]                (forward)
//                         = w[ch*16+8*h+cc][g*TF+fl][taps-1-t]         (backward-data: roles swapped, taps reversed)
__global__ void __launch_bounds__(kThreads)
gb_weight_prep_kernel(const float *__restrict__ w, bf16 *__restrict__ wt, int K, int C, int taps, int NC, int TF,
                      int n_fgrp, int flip)
{
    const long total = (long)n_fgrp * NC * taps * TF * CK;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int cc = (int)(idx % 8);
    const int fl = (int)((idx / 8) % TF);
    const int h = (int)((idx / (8L * TF)) % 2);
    const int t = (int)((idx / ((long)CK * TF)) % taps);
    const int ch = (int)((idx / ((long)CK * TF * taps)) % NC);
    const int g = (int)(idx / ((long)CK * TF * taps * NC));
    const int f = g * TF + fl, c = ch * CK + 8 * h + cc;
    float v = 0.f;
    if (!flip) {
        if (f < K && c < C) v = w[((long)f * C + c) * taps + t];
    } else {
        if (f < C && c < K) v = w[((long)c * C + f) * taps + (taps - 1 - t)];
    }
    wt[idx] = f32_to_bf16(v);
}

// QN > 0 (maps with an even number of columns): an item is four neighbouring pixels whose first
// lies at a map column that is a multiple of four, for one channel half; QN such items per thread
// at most.  Every row of a plane starts at an even element, so the 8-byte load is 4-byte aligned.
// Tile column c lies at LDS column c + par, where par = (first map column of the tile) mod 4.
// QN = 0: single pixels, 2-byte loads.
// KH > 0: the kernel has KH tap rows (compile time, operands shared between tap rows as described
// at the top); KH = 0: any number, four operand reads per tap.
template <typename TO, int WM, int QN, int KH>
__global__ void __launch_bounds__(kThreads, 2)
gemm_conv_bf16_kernel(GbParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int TF = WM * 32, NI = QN ? QN : kItems;
    unsigned char *xs = smem;                  // [2][rows][cols_p] pieces of 8 channels
    unsigned char *wsm = smem + p.xs_bytes;    // [taps][2][TF] pieces of 8 channels

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

    // Item it = tid + 256*i: channel half g = it / n_pix, item it % n_pix of the tile.  voff[i] is where
    // channel 8*g of the chunk is read for the item's (first) pixel, relative to the chunk's first channel;
    // items outside the map (and the padding of the item list) read offset 0, which is a valid address.
    // lds[i]: byte offset of the item's (first) pixel in the tile.  `zero`: bit 4*i + m says that pixel m of
    // item i lies outside the map (its value is replaced by zero where the call needs that; quad form), bit 16 + i that
    // the whole item does, bit 24 + i that the item is padding of the list (not written).
    const int par = QN ? (v0 - p.off_w) & 3 : 0;
    const int mc0 = v0 - p.off_w - par;        // map column of LDS column 0
    unsigned voff[NI];
    int lds[NI];
    unsigned zero = 0;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int it = tid + i * kThreads;
        const int g = it >= p.n_pix ? 1 : 0, pi = it - g * p.n_pix;
        const bool listed = it < 2 * p.n_pix;
        const int per_row = QN ? p.gpr : p.cols;
        const int r = pi / per_row, c = (QN ? 4 : 1) * (pi - r * per_row);
        const int irow = u0 + r * p.d - p.off_h, icol = mc0 + c;
        const bool ok = listed && irow >= 0 && irow < p.Hin && icol >= 0 && icol < p.Win;
        voff[i] = ok ? (unsigned)(8 * g) * HW + (unsigned)(irow * p.Win + icol) : 0u;
        lds[i] = ((g * p.rows + r) * p.cols_p + c) * 16;
        if (QN) {
#pragma unroll
            for (int m = 0; m < 4; ++m) zero |= ok && icol + m < p.Win ? 0u : 1u << (4 * i + m);
        }
        zero |= ok ? 0u : 1u << (16 + i);
        zero |= listed ? 0u : 1u << (24 + i);
    }
    // does any pixel of this tile have to be replaced by zero?  (the same for all threads)
    const bool masks = p.zero_fill && !(u0 - p.off_h >= 0 && u0 + (p.rows - 1) * p.d - p.off_h < p.Hin && mc0 >= 0 &&
                                       mc0 + p.cols_p <= p.Win);

    f32x16 acc[WM][4];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[wm][j][i] = 0.f;

    constexpr int XW = QN ? 2 : 1;
    unsigned xr[NI][8][XW];      // channel j of the item: four pixels (two words), or one 2-byte value
    u32x4 wv[kWq];
    // Every load is issued unconditionally: a load under a condition would be waited for on the spot.
    auto fetch = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * CK;
        auto load = [&](int i, int j, unsigned off, unsigned plane_off) __attribute__((always_inline)) {
            if constexpr (QN) {
                const u32x2 q = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(off * 2u), (int)(plane_off * 2u), 0));
                xr[i][j][0] = q[0]; xr[i][j][1] = q[1];
            } else {
                xr[i][j][0] = __builtin_amdgcn_raw_buffer_load_b16(rx, (int)(off * 2u), (int)(plane_off * 2u), 0);
            }
        };
        if (c0 + CK <= p.Cin) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) load(i, j, voff[i], (unsigned)(c0 + j) * HW);
        } else {
            // last chunk of a padded channel count: channels at or beyond Cin meet zero weights; the chunk's
            // first channel is read instead so that the value is a finite one from inside the tensor
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int g8 = tid + i * kThreads >= p.n_pix ? 8 : 0;
                const unsigned pix = voff[i] - (unsigned)g8 * HW * ((zero >> (16 + i)) & 1u ? 0u : 1u);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    load(i, j, c0 + g8 + j < p.Cin ? voff[i] + (unsigned)j * HW : pix, (unsigned)c0 * HW);
            }
        }
        const bf16 *wsrc = p.wt + ((long)fg * p.NC + ch) * taps * TF * CK;
        const BufRsrc rw = buf_rsrc(wsrc, wsrc + (long)taps * TF * CK);      // the padding of the LDS part reads zero
#pragma unroll
        for (int q = 0; q < kWq; ++q)
            wv[q] = __builtin_amdgcn_raw_buffer_load_b128(rw, (q * kThreads + tid) * 16, 0, 0);
    };

    // per-lane LDS addresses: B = (channel half hi, row R0, column cb*32 + lo), A = (half hi, filter lo)
    const int R0 = 4 * (wave >> 1), cb = wave & 1;
    const unsigned char *xlane = xs + ((hi * p.rows + R0) * p.cols_p + cb * 32 + lo + par) * 16;
    const unsigned char *wlane = wsm + (hi * TF + lo) * 16;
    const int rowb = p.cols_p * 16;

    fetch(0);
    for (int ch = 0; ch < p.NC; ++ch) {
        __syncthreads();      // every wave is done reading the previous chunk
        // The loaded values are combined here, not where they were fetched: combined early (which the
        // compiler would do where it saves registers) every load is waited for on the spot, and a chunk
        // then costs many memory round trips instead of one.
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int x = 0; x < XW; ++x) asm volatile("" : "+v"(xr[i][j][x]));
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (i < p.n_items && !((zero >> (24 + i)) & 1u)) {
                if constexpr (QN) {
                    u32x4 o[4];      // pixel m: the low / high halves of word m/2 of the eight channels
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        o[0][k] = __builtin_amdgcn_perm(xr[i][2 * k + 1][0], xr[i][2 * k][0], 0x05040100u);
                        o[1][k] = __builtin_amdgcn_perm(xr[i][2 * k + 1][0], xr[i][2 * k][0], 0x07060302u);
                        o[2][k] = __builtin_amdgcn_perm(xr[i][2 * k + 1][1], xr[i][2 * k][1], 0x05040100u);
                        o[3][k] = __builtin_amdgcn_perm(xr[i][2 * k + 1][1], xr[i][2 * k][1], 0x07060302u);
                    }
                    if (masks) {
#pragma unroll
                        for (int m = 0; m < 4; ++m)
                            if ((zero >> (4 * i + m)) & 1u) o[m] = u32x4{0u, 0u, 0u, 0u};
                    }
#pragma unroll
                    for (int m = 0; m < 4; ++m) *(u32x4 *)(xs + lds[i] + 16 * m) = o[m];
                } else {
                    const bool z = masks && ((zero >> (16 + i)) & 1u);
                    u32x4 v;
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = z ? 0u : xr[i][2 * k][0] | (xr[i][2 * k + 1][0] << 16);
                    *(u32x4 *)(xs + lds[i]) = v;
                }
            }
#pragma unroll
        for (int q = 0; q < kWq; ++q)
            if (q < p.n_wq) ((u32x4 *)wsm)[q * kThreads + tid] = wv[q];
        __syncthreads();
        fetch(ch + 1 < p.NC ? ch + 1 : ch);      // in flight while the matrix cores run (the last one is not used)

        // ---- matrix cores: one instruction per tap and accumulator tile, k = the chunk's 16 channels
        for (int tb = 0; tb < p.kw; ++tb) {
            const unsigned char *xb = xlane + tb * p.d * 16;
            const unsigned char *wb = wlane + tb * 2 * TF * 16;
            if constexpr (KH > 0) {
                bf16x8 A[KH][WM];
#pragma unroll
                for (int ta = 0; ta < KH; ++ta)
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm)
                        A[ta][wm] = *(const bf16x8 *)(wb + ta * p.kw * 2 * TF * 16 + wm * 32 * 16);
#pragma unroll
                for (int r = 0; r < KH + 3; ++r) {
                    const bf16x8 B = *(const bf16x8 *)(xb + r * rowb);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int ta = r - j;
                        if (ta >= 0 && ta < KH) {
#pragma unroll
                            for (int wm = 0; wm < WM; ++wm)
                                acc[wm][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ta < 0 || ta >= KH ? 0 : ta][wm], B, acc[wm][j], 0, 0, 0);
                        }
                    }
                }
            } else {
                for (int ta = 0; ta < p.kh; ++ta) {
                    bf16x8 A[WM], B[4];
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm) A[wm] = *(const bf16x8 *)(wb + ta * p.kw * 2 * TF * 16 + wm * 32 * 16);
#pragma unroll
                    for (int j = 0; j < 4; ++j) B[j] = *(const bf16x8 *)(xb + (ta + j) * rowb);
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[wm][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[wm], B[j], acc[wm][j], 0, 0, 0);
                }
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
    // stores through a descriptor of this image's filter block: one scalar offset per filter, no 64-bit
    // address arithmetic per output
    const BufRsrc ro = buf_rsrc(out_n, out_n + (long)(f_left < TF ? f_left : TF) * plane);
    const bool all_f = f_left >= TF;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = u0 + (R0 + j) * p.d;
        const int col = v0 + cb * 32 + lo;
        if (row >= p.Hout || col >= p.Wout) continue;
        const unsigned o = (unsigned)(row * p.Wout + col) + (hi ? 4u * (unsigned)plane : 0u);
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int fl = wm * 32 + 8 * (i / 4) + (i % 4);
                if (all_f || fl + 4 * hi < f_left)
                    buf_st(ro, (TO *)nullptr, o, (unsigned)fl * (unsigned)plane, act_apply(p.act, acc[wm][j][i] + bv[wm][i]));
            }
        }
    }
}

struct GbPlan {
    bool ok;
    int WM, TF, NC, rows, cols, cols_p, gpr, n_pix, n_items, qn, n_wq, xs_bytes, n_fgrp, n_rowtile, n_coltile, nrb, full_cls;
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
    // groups of four pixels on the map's four-column grid: the tile begins 0-3 columns into its first group
    g.gpr = (g.cols + 3 + 3) / 4;
    g.qn = 0;
    if (Win % 2 == 0) {
        const int items = (2 * g.rows * g.gpr + kThreads - 1) / kThreads;
        g.qn = items <= 2 ? 2 : items <= 4 ? 4 : 0;
    }
    if (g.qn) {
        g.cols_p = 4 * g.gpr;
        g.n_pix = g.rows * g.gpr;
    } else {
        g.cols_p = g.cols;
        g.n_pix = g.rows * g.cols;
    }
    g.n_items = (2 * g.n_pix + kThreads - 1) / kThreads;
    if (g.n_items > (g.qn ? g.qn : kItems)) return g;
    g.xs_bytes = (2 * g.rows * g.cols_p * 16 + 255) & ~255;
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
    if ((g.tiles + kXcds - 1) / kXcds * kXcds > 0x7fffffffL) return g;      // the grid: such calls take the other kernels
    g.ok = true;
    return g;
}

template <typename TO, int WM, int QN>
static void gb_launch_kh(const GbParams &p, unsigned grid, size_t lds, hipStream_t st)
{
    switch (p.kh) {
    case 3: gemm_conv_bf16_kernel<TO, WM, QN, 3><<<dim3(grid), dim3(kThreads), lds, st>>>(p); break;
    case 4: gemm_conv_bf16_kernel<TO, WM, QN, 4><<<dim3(grid), dim3(kThreads), lds, st>>>(p); break;
    case 5: gemm_conv_bf16_kernel<TO, WM, QN, 5><<<dim3(grid), dim3(kThreads), lds, st>>>(p); break;
    default: gemm_conv_bf16_kernel<TO, WM, QN, 0><<<dim3(grid), dim3(kThreads), lds, st>>>(p); break;
    }
}

template <typename TO, int WM>
static void gb_launch_qn(const GbParams &p, int qn, unsigned grid, size_t lds, hipStream_t st)
{
    if (qn == 2) gb_launch_kh<TO, WM, 2>(p, grid, lds, st);
    else if (qn == 4) gb_launch_kh<TO, WM, 4>(p, grid, lds, st);
    else gb_launch_kh<TO, WM, 0>(p, grid, lds, st);
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
    p.zero_fill = off ? 1 : 0;
    p.NC = g.NC; p.rows = g.rows; p.cols = g.cols; p.cols_p = g.cols_p; p.gpr = g.gpr; p.n_pix = g.n_pix;
    p.n_items = g.n_items;
    p.n_wq = g.n_wq;
    p.xs_bytes = g.xs_bytes;
    p.n_rowtile = g.n_rowtile; p.n_coltile = g.n_coltile; p.n_fgrp = g.n_fgrp; p.nrb = g.nrb; p.full_cls = g.full_cls;
    p.tiles = g.tiles;
    p.per_xcd = (g.tiles + kXcds - 1) / kXcds;
    const unsigned grid = (unsigned)(p.per_xcd * kXcds);
    if (tout == DSK_BF16) {
        if (g.WM == 2) gb_launch_qn<bf16, 2>(p, g.qn, grid, g.lds_bytes, st);
        else gb_launch_qn<bf16, 1>(p, g.qn, grid, g.lds_bytes, st);
    } else {
        if (g.WM == 2) gb_launch_qn<float, 2>(p, g.qn, grid, g.lds_bytes, st);
        else gb_launch_qn<float, 1>(p, g.qn, grid, g.lds_bytes, st);
    }
    return check_launch();
}

// ---- entry points for the dispatcher (bf16 input maps only)
// a 1 x 1 kernel has no taps to space: its tiles take neighbouring rows
static int tap_spacing(const ConvShape &s) { return s.kh == 1 && s.kw == 1 ? 1 : s.d; }

size_t conv_bf16_ws_bytes(int which, const ConvShape &s)
{
    const GbPlan g = which == DSK_WS_CONV_FWD ? gb_plan(s.N, s.C, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, tap_spacing(s))
                                              : gb_plan(s.N, s.K, s.Wo, s.C, s.H, s.W, s.kh, s.kw, tap_spacing(s));
    return g.ok ? g.wt_bytes : 0;
}

bool conv_bf16_supported(int which, const ConvShape &s)
{
    if ((long)s.H * s.W >= (1L << 28) || (long)s.C * s.H * s.W >= (1L << 30) ||
        (long)s.K * s.Ho * s.Wo >= (1L << 30))
        return false;
    if (which == DSK_WS_CONV_FWD) return gb_plan(s.N, s.C, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, tap_spacing(s)).ok;
    if (which == DSK_WS_CONV_BWD_DATA) return gb_plan(s.N, s.K, s.Wo, s.C, s.H, s.W, s.kh, s.kw, tap_spacing(s)).ok;
    return false;
}

int launch_conv_fwd_bf16(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                         dsk_dtype out, int act, void *ws, hipStream_t st)
{
    return gb_run(x, y, w, b, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, tap_spacing(s), 0, act, 0, s.K, s.C, out, ws, st);
}

int launch_conv_bwd_data_bf16(const void *dy, const float *w, void *dx, const ConvShape &s, dsk_dtype out, void *ws,
                              hipStream_t st)
{
    return gb_run(dy, dx, w, nullptr, s.N, s.K, s.Ho, s.Wo, s.C, s.H, s.W, s.kh, s.kw, tap_spacing(s), 1, DSK_ACT_NONE, 1,
                  s.K, s.C, out, ws, st);
}

} // namespace dsk
