// Matrix-core (MFMA) kernels for the sparse-kernel convolution operators on gfx950:
// forward and backward-data (paper Sec. 3.1-3.2, Sec. 4.1: delta_k = pad(delta_{k+1})
// *^1 rot180(W_{k,d})) share one implicit-GEMM kernel; backward-weight (Sec. 4.1:
// grad W_{k,d} = x_k *^1 rot(delta_{k+1,d})) has its own.
//
// No column matrix is ever materialised (the paper gathers the non-zero taps into
// one; here the gather happens on the way from LDS to the matrix cores).
//
// Tiling idea, common to both kernels: a workgroup's output ROWS all lie in one
// residue class modulo the spacing d (rows u0, u0+d, u0+2d, ...), while its COLUMNS
// are contiguous.  The kh taps of such rows hit input rows of the same class, so a
// tile of TH rows needs only TH+kh-1 input rows whatever d is, and every global
// load is a contiguous row segment.  The column halo is (kw-1)*d.
//
// fp32 path: v_mfma_f32_32x32x2_f32.  Lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; register r of the 16 results holds D[8*(r/4) + 4*(l/32) + r%4][l%32].
#include <atomic>

#include "dsk_internal.h"

namespace dsk {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

static constexpr int kThreads = 256;
static constexpr int kXcds = 8;
static constexpr size_t kMaxLds = 64 * 1024;      // forward / backward-data: two workgroups per CU
static constexpr size_t kMaxLdsBw = 76 * 1024;    // backward-weight: still two per CU (160 KB)

// Dynamic LDS beyond the default limit has to be enabled per kernel (and device): done the first
// time a kernel needs that much, not on every launch.
template <auto Kernel>
static void allow_lds(size_t bytes)
{
    static std::atomic<size_t> granted[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
    if (dev >= 0 && granted[dev].load(std::memory_order_acquire) >= bytes) return;
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)bytes);
    if (dev >= 0) granted[dev].store(bytes, std::memory_order_release);
}


// ============================================================================
// forward / backward-data: out[n][f][u][v] = epi( sum_{c,a,b} wt[c][a][b][f] *
//                                   in[n][c][u + a*d - off][v + b*d - off] ), in = 0 outside
// ============================================================================
static constexpr int TH = 8;    // output rows per workgroup (one residue class mod d)
static constexpr int TW = 64;   // output columns per workgroup

// A rectangle of the output map covered by tiles of one shape: 4*nr rows of a residue class by 32*nh columns
// (nr, nh = 1 or 2).  The whole map is one rectangle of 8 x 64 tiles unless its last tiles would be at most half
// full: then the last strip of rows and / or columns is a rectangle of its own with tiles of half the height or
// width, so that the matrix cores do not spend a whole tile on it.
struct GcRegion {
    int nr, nh;
    int u_base, v_base;              // first row / column of the rectangle
    int rows, cols, chan_stride;     // LDS tile: 4*nr+kh-1 by 32*nh+(kw-1)*d
    unsigned m_cs, m_cols;           // 2^32 / chan_stride + 1 and 2^32 / cols + 1: e / x = mulhi(e, m) for the small e of the tile index
    int n_xi;                        // input-tile floats per thread and chunk
    int n_rowtile, n_coltile;
    int nrb, full_cls;               // row blocks of d*4*nr rows; residue classes that have a tile in the last one (the others: nrb-1 tiles)
    long tiles;                      // N * n_rowtile * n_coltile * n_fgrp
    long first_block, per_xcd;       // physical workgroups [first_block, first_block + 8*per_xcd) take these tiles
};

struct GcParams {
    const void *in;
    void *out;
    const float *wt;     // [n_fgrp][Cpad][taps][TF], zero padded
    const float *bias;   // may be null
    float *partial;      // split tiles: [2 * n_wg][WM * 64][256] raw accumulators
    int N, Cin, Hin, Win, Fout, Hout, Wout;      // Fout: the filters of this launch (`out` and `bias` begin at its first)
    int Fimg;            // filter planes per image of `out`
    int kh, kw, d, off_h, off_w, act;
    int Cpad, Cc, NC;    // padded channel count, channels per LDS chunk (even), chunks per tile
    int xs_floats;       // Cc*chan_stride of the largest tile shape rounded up to a multiple of 256
    int n_wi;            // weight float4s per thread and chunk (the LDS part is padded)
    int n_fgrp;
    GcRegion reg[4];     // reg[0] alone when the workgroups are persistent (split tiles)
    int n_reg;
    long tiles;          // output tiles of reg[0] (persistent workgroups)
    int rounds;          // persistent workgroups: whole tiles each of them takes first
    int rem_units;       // (tiles - rounds * n_wg) * NC: chunks of the tiles left after that
    long n_wg, per_xcd;  // logical workgroups; the grid is per_xcd * 8
    // how the input's planes are found (video layers; see ConvShape): image n at slot n + n / bgroup * bskip,
    // in_bstride elements per slot, channel v a further v*Hin*Win + v / gsize * gjump; in_extent readable elements
    int gsize, bgroup, bskip;
    long gjump, in_bstride, in_extent;
};

// Weight layout transform.  flip = 0: wt[g][c][t][fl] = w[g*TF+fl][c][t]            (forward)
//                           flip = 1: wt[g][k][t][cl] = w[k][g*TF+cl][taps-1-t]     (backward-data)
__global__ void __launch_bounds__(kThreads)
gc_weight_prep_kernel(const float *__restrict__ w, float *__restrict__ wt, int K, int C, int taps,
                      int Cpad, int TF, int n_fgrp, int flip, int round_bf16, int f0, int f_end)
{
    const long total = (long)n_fgrp * Cpad * taps * TF;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int fl = (int)(idx % TF);
    const int t = (int)((idx / TF) % taps);
    const int c = (int)((idx / ((long)TF * taps)) % Cpad);
    const int g = (int)(idx / ((long)TF * taps * Cpad));
    const int f = f0 + g * TF + fl;      // (a launch may cover the outputs f0 .. f_end-1 only)
    float v = 0.f;
    if (!flip) {
        if (f < f_end && c < C) v = w[((long)f * C + c) * taps + t];
    } else {
        // channel index of the GEMM is the filter k of w, output index is the channel c of w
        if (f < f_end && c < K) v = w[((long)c * C + f) * taps + (taps - 1 - t)];
    }
    wt[idx] = round_bf16 ? bf16_to_f32(f32_to_bf16(v)) : v;
}

// tile index -> filter group, image, first output row (of its residue class), first column
__device__ inline void gc_decode_tile(const GcParams &p, const GcRegion &g, long tile, int &fg, int &n, int &u0, int &v0)
{
    fg = (int)(tile % p.n_fgrp); tile /= p.n_fgrp;
    const int ct = (int)(tile % g.n_coltile); tile /= g.n_coltile;
    const int rt = (int)(tile % g.n_rowtile);
    n = (int)(tile / g.n_rowtile);
    // Row tiles are numbered class by class, down the map within a class: tiles that follow each other
    // (and run on one XCD at the same time) then share input rows and columns.  Numbered row block by
    // row block, neighbours would be different residue classes, which share no input row.
    const int nf = g.full_cls * g.nrb;
    int cls, rb;
    if (rt < nf) {
        cls = rt / g.nrb; rb = rt - cls * g.nrb;
    } else {
        const int q = (rt - nf) / (g.nrb - 1);
        cls = g.full_cls + q; rb = rt - nf - q * (g.nrb - 1);
    }
    u0 = g.u_base + rb * p.d * 4 * g.nr + cls;
    v0 = g.v_base + ct * 32 * g.nh;
}

// bias, non-linearity, store; 32 consecutive pixels per filter per store instruction.
// Register i of a lane belongs to filter 8*(i/4) + (i%4) + 4*hi of its 32-filter block: the
// two candidates are uniform over the wave, so their biases come through scalar loads.
template <typename TO, int WM, int NR, int NH>
__device__ inline void gc_epilogue(const GcParams &p, const f32x16 (&acc)[WM][NR * NH], int fg, int n, int u0, int v0,
                                   int wave, int lo, int hi)
{
    constexpr int TF = WM * 32;
    const long plane = (long)p.Hout * p.Wout;
    TO *out_n = (TO *)p.out + ((long)n * p.Fimg + (long)fg * TF) * plane;
    const int f_left = p.Fout - fg * TF;      // filters of this group that exist
    // The biases of this lane's filters, fetched together BEFORE the first store.  Loaded where
    // they are used, each load has to be waited for on the spot (it may not pass the stores
    // before it: `out` could alias `bias`), and a tile's 64-128 outputs per lane then cost as
    // many memory round trips.  Filters beyond Fout read zero through the descriptor's range.
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
    for (int wn = 0; wn < NR * NH; ++wn) {
        const int row = u0 + (NR * wave + wn / NH) * p.d;
        const int col = v0 + (wn % NH) * 32 + lo;
        if (row >= p.Hout || col >= p.Wout) continue;
        TO *o = out_n + (long)row * p.Wout + col + (hi ? 4 * plane : 0);
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int fl = wm * 32 + 8 * (i / 4) + (i % 4);      // filter of the hi = 0 lanes
                if (fl + 4 * hi < f_left) stf(o, (long)fl * plane, act_apply(p.act, acc[wm][wn][i] + bv[wm][i]));
            }
        }
    }
}

// XI / WI: upper bounds of what one thread stages per chunk: input-tile elements
// (Cc*chan_stride <= 256*XI) and weight float4s (Cc*taps*TF <= 1024*WI).
//
// Work distribution.  SPLIT = false: logical workgroup g owns tile g.  SPLIT = true (chosen
// by the host when the tile count is not a comfortable multiple of what the chip holds at
// once): n_wg persistent workgroups first take `rounds` whole tiles each, round r giving
// tile r*n_wg + g to workgroup g, so that workgroups running side by side work on
// neighbouring tiles and share their input through the L2.  The channel chunks of the
// tiles left over (fewer than n_wg) are numbered tile-major and workgroup g takes chunks
// [g*U/n_wg, (g+1)*U/n_wg) of these U, so the shares differ by one chunk at most and every
// XCD stays busy.  Such a range may begin or end inside a tile; a piece of a tile is
// written as raw accumulators to `partial`, and gc_fixup_kernel adds the pieces of every
// left-over tile in a fixed order and applies the epilogue.
//
// With fewer tiles than workgroups (small maps) `rounds` is 0 and the workgroups share the chunks of all
// tiles.
//
// Pipeline: the global loads of chunk t+1 are issued before the matrix cores start on chunk
// t and land in registers meanwhile; they are written to LDS after chunk t is done.
//
// NR, NH: shape of the tiles of rectangle g (4*NR rows by 32*NH columns); a wave owns rows NR*wave .. NR*wave+NR-1
// of the tile and all its columns.  wg: the logical workgroup (persistent ones: of the launch; else: of g).
// KW: taps per kernel row when known at compile time (0: p.kw), so that the row of taps is unrolled and the LDS
// reads of the next tap are issued under the matrix instructions of the current one.
template <typename TI, typename TO, int WM, int XI, int WI, bool SPLIT, int NR, int NH, int KW = 0>
__device__ __forceinline__ void gc_body(const GcParams &p, const GcRegion &g, const long wg, float *smem)
{
    constexpr int TF = WM * 32;
    float *xs = smem;                   // [Cc][rows][cols]
    float *wsm = smem + p.xs_floats;    // [Cc][taps][TF]

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    int round = 0;
    int ub = (int)wg * p.rem_units / (int)p.n_wg;      // rem_units * n_wg < 2^31 by the host's choice
    const int ue = ((int)wg + 1) * p.rem_units / (int)p.n_wg;

    const unsigned HW = (unsigned)(p.Hin * p.Win);   // Cin*Hin*Win < 2^30 is checked on the host
    const int taps = p.kh * p.kw;
    const int n4 = p.Cc * taps * TF / 4;

    bool first_piece = true;
    for (;;) {
        // Everything derived from the lane index is derived again for every tile: carried
        // across tiles it would take registers the accumulators and the prefetch need.
        int tid = threadIdx.x;
        if (SPLIT) asm volatile("" : "+v"(tid));
        const int lane = tid & 63, lo = lane & 31, hi = lane >> 5;
        // per-lane LDS bases; the k-step offsets are uniform over the wave
        const float *xlane = xs + hi * g.chan_stride + (NR * wave) * g.cols + lo;
        const float *wlane = wsm + hi * taps * TF + lo;
        long tile = wg;
        int cb = 0, ce = p.NC;
        if (SPLIT) {
            if (round < p.rounds) {
                tile = round * p.n_wg + wg;
            } else {
                if (ub >= ue) break;
                const int lt = ub / p.NC;
                tile = p.rounds * p.n_wg + lt;
                cb = ub - lt * p.NC;
                ce = cb + (ue - ub) < p.NC ? cb + (ue - ub) : p.NC;
            }
        }
        int fg, n, u0, v0;
        gc_decode_tile(p, g, tile, fg, n, u0, v0);
        const TI *in_n = (const TI *)p.in + (p.bgroup ? n + (long)(n / p.bgroup) * p.bskip : (long)n) * p.in_bstride;
        const TI *in_end = (const TI *)p.in + p.in_extent;

        // Where this thread's share of the input tile comes from; the same for every chunk:
        // element e = tid + 256*i of the LDS tile [Cc][rows][cols] (padded to a multiple of 256)
        // is read at voff[i] floats beyond the first channel of the chunk.  Elements outside
        // the map, or in the padding, are read from offset 0 instead, which is always a valid
        // address, and bit i of `zero` says that the tile gets 0 there.
        // Where no zeroing is needed when the tile is written to LDS (uniform).  Forward: a tile entry outside the
        // map only feeds outputs outside the output map, which are not stored.  Backward-data: tiles that lie wholly
        // inside the error map.  (Channels beyond Cin meet zero weights, and the padding at the end of the LDS tile
        // is never read.)
        const bool no_zeroing = (p.off_h == 0 && p.off_w == 0) ||
                                (u0 - p.off_h >= 0 && u0 - p.off_h + (g.rows - 1) * p.d < p.Hin &&
                                 v0 - p.off_w >= 0 && v0 - p.off_w + g.cols <= p.Win);
        // QUAD (fp32 maps, tiles a multiple of four columns wide, whole chunks, no zeroing): a thread stages FOUR
        // neighbouring columns per load (16 bytes, any alignment) and LDS write instead of one -- the vector memory
        // path spends as long on a wave's 4-byte loads as on its 16-byte ones.  Item tid + 256*i holds elements
        // 4*item .. 4*item+3 of the tile; columns beyond the map read what follows in memory (finite values of the
        // map, or zero beyond the tensor), which only feed outputs that are not stored.
        constexpr bool QUADX = sizeof(TI) == 4 && XI % 4 == 0;
        const bool quad = QUADX && no_zeroing && g.cols % 4 == 0 && p.Cpad == p.Cin && (!p.gsize || p.gsize % p.Cc == 0);
        unsigned voff[XI];
        unsigned zero = 0;
        {
            const int n_x = p.Cc * g.chan_stride;
            const int row0 = u0 - p.off_h, col0 = v0 - p.off_w;
            if (quad) {
#pragma unroll
                for (int i = 0; i < XI / 4; ++i) {
                    const int e = 4 * (tid + i * kThreads);
                    const int c = (int)__umulhi((unsigned)e, g.m_cs), rem = e - c * g.chan_stride;
                    const int r = (int)__umulhi((unsigned)rem, g.m_cols), col = rem - r * g.cols;
                    voff[i] = e < n_x ? (unsigned)c * HW + (unsigned)((row0 + r * p.d) * p.Win + col0 + col) : 0u;
                }
            } else {
#pragma unroll
            for (int i = 0; i < XI; ++i) {
                const int e = tid + i * kThreads;
                // (exact: e * chan_stride and rem * cols stay below 2^32; a division costs some 40 instructions)
                const int c = (int)__umulhi((unsigned)e, g.m_cs), rem = e - c * g.chan_stride;
                const int r = (int)__umulhi((unsigned)rem, g.m_cols), col = rem - r * g.cols;
                const int irow = row0 + r * p.d, icol = col0 + col;
                const bool ok = e < n_x && irow >= 0 && irow < p.Hin && icol >= 0 && icol < p.Win;
                voff[i] = ok ? (unsigned)c * HW + (unsigned)(irow * p.Win + icol) : 0u;
                zero |= ok ? 0u : 1u << i;
            }
            }
        }

        f32x16 acc[WM][NR * NH];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm)
#pragma unroll
            for (int wn = 0; wn < NR * NH; ++wn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[wm][wn][i] = 0.f;

        float xv[XI];
        f32x4 wv[WI];
        // Every load is issued unconditionally (padding reads offset 0): a load under a
        // condition makes the compiler wait for it right away to merge the two values.
        auto fetch = [&](int c0) __attribute__((always_inline)) {
            const int g0 = p.gsize ? c0 / p.gsize : 0;      // the channel group the chunk begins in
            const TI *src = in_n + (long)c0 * (long)HW + g0 * p.gjump;
            const BufRsrc rx = buf_rsrc(src, in_end);
            if (QUADX && quad) {
#pragma unroll
                for (int i = 0; i < XI / 4; ++i) {
                    const f32x4 q = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(voff[i] * 4u), 0, 0));
#pragma unroll
                    for (int j = 0; j < 4; ++j) xv[4 * i + j] = q[j];
                }
            } else if (c0 + p.Cc <= p.Cin && (!p.gsize || c0 - g0 * p.gsize + p.Cc <= p.gsize)) {
#pragma unroll
                for (int i = 0; i < XI; ++i) xv[i] = buf_ld(rx, src, voff[i], 0u);
            } else {
                // Last chunk of a padded channel count: channels beyond Cin meet zero weights; read the
                // chunk's first channel instead so the address stays inside the tensor.  A chunk that
                // straddles channel groups: the later group's planes lie gjump elements further on
                // (the host checks that this stays below 2^30 elements).
#pragma unroll
                for (int i = 0; i < XI; ++i) {
                    unsigned v = voff[i];
                    if (!((zero >> i) & 1u)) {
                        const unsigned cl = __umulhi((unsigned)(tid + i * kThreads), g.m_cs);      // the element's channel
                        const int cv = c0 + (int)cl;
                        if (cv >= p.Cin) v -= cl * HW;
                        else if (p.gsize) v += (unsigned)(cv / p.gsize - g0) * (unsigned)p.gjump;
                    }
                    xv[i] = buf_ld(rx, src, v, 0u);
                }
            }
            // the descriptor ends with the chunk's weights: the padding of the LDS part reads zero
            const float *wsrc = p.wt + ((long)fg * p.Cpad + c0) * taps * TF;
            const BufRsrc rw = buf_rsrc(wsrc, wsrc + 4 * n4);
#pragma unroll
            for (int q = 0; q < WI; ++q)
                wv[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, (q * kThreads + tid) * 16, 0, 0));
        };

        fetch(cb * p.Cc);
        for (int ch = cb; ch < ce; ++ch) {
            __syncthreads();      // every wave is done reading the previous chunk
            if (QUADX && quad) {
#pragma unroll
                for (int i = 0; i < XI / 4; ++i)
                    if (4 * (tid + i * kThreads) < p.xs_floats) {      // (the LDS part of the tile ends there)
                        const f32x4 q = {xv[4 * i], xv[4 * i + 1], xv[4 * i + 2], xv[4 * i + 3]};
                        ((f32x4 *)xs)[tid + i * kThreads] = q;
                    }
            } else if (no_zeroing) {
#pragma unroll
                for (int i = 0; i < XI; ++i)
                    if (i < g.n_xi) xs[tid + i * kThreads] = xv[i];
            } else {
#pragma unroll
                for (int i = 0; i < XI; ++i)
                    if (i < g.n_xi) xs[tid + i * kThreads] = (zero >> i) & 1u ? 0.f : xv[i];
            }
#pragma unroll
            for (int q = 0; q < WI; ++q)
                if (q < p.n_wi) ((f32x4 *)wsm)[q * kThreads + tid] = wv[q];
            __syncthreads();
            if (ch + 1 < ce) fetch((ch + 1) * p.Cc);      // in flight while the matrix cores run

            // ---- matrix cores: k index = (channel pair, tap); lanes 32..63 take the odd channel
            for (int cp = 0; cp < p.Cc; cp += 2) {
                const float *xb = xlane + cp * g.chan_stride;
                const float *wb = wlane + cp * taps * TF;
                auto tap = [&](int ta, int tb, int kw) __attribute__((always_inline)) {
                    const int xo = ta * g.cols + tb * p.d, wo = (ta * kw + tb) * TF;
                    float A[WM], B[NR * NH];
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm) A[wm] = wb[wo + wm * 32];
#pragma unroll
                    for (int wn = 0; wn < NR * NH; ++wn) B[wn] = xb[xo + (wn / NH) * g.cols + (wn % NH) * 32];
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                        for (int wn = 0; wn < NR * NH; ++wn)
                            acc[wm][wn] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[wm], B[wn], acc[wm][wn], 0, 0, 0);
                };
                if constexpr (KW > 0) {      // (square kernels: the host launches these instances for kh = kw only)
#pragma unroll
                    for (int ta = 0; ta < KW; ++ta)
#pragma unroll
                        for (int tb = 0; tb < KW; ++tb) tap(ta, tb, KW);
                } else {
                    for (int ta = 0; ta < p.kh; ++ta)
                        for (int tb = 0; tb < p.kw; ++tb) tap(ta, tb, p.kw);
                }
            }
        }

        if (!SPLIT || (cb == 0 && ce == p.NC)) {
            gc_epilogue<TO, WM, NR, NH>(p, acc, fg, n, u0, v0, wave, lo, hi);
        } else {
            // a piece of a split tile: slot 2g holds the piece a range begins with, 2g+1 the one it ends with
            float *slot = p.partial + (2 * wg + (first_piece ? 0 : 1)) * (long)(WM * 64 * kThreads);
#pragma unroll
            for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                for (int wn = 0; wn < NR * NH; ++wn)
#pragma unroll
                    for (int i = 0; i < 16; ++i) slot[((wm * 4 + wn) * 16 + i) * kThreads + tid] = acc[wm][wn][i];
        }
        if (!SPLIT) break;
        if (round < p.rounds) {
            ++round;
        } else {
            ub += ce - cb;
            first_piece = false;
        }
    }
}

// HALF: the launch may hold rectangles with tiles of half the height or width (instances for them exist only
// where the host uses them: one tile per workgroup, ordinary halos).
template <typename TI, typename TO, int WM, int XI, int WI, bool SPLIT, bool HALF, int KW = 0>
__global__ void __launch_bounds__(kThreads, 2)
gemm_conv_kernel(GcParams p)
{
    extern __shared__ __align__(16) float smem[];
    // consecutive physical workgroups go to different XCDs; give each XCD one contiguous
    // run of logical workgroups so that neighbours (shared halo, same input tile) share an L2
    if constexpr (SPLIT) {
        const long wg = (long)(blockIdx.x % kXcds) * p.per_xcd + blockIdx.x / kXcds;
        if (wg >= p.n_wg) return;
        gc_body<TI, TO, WM, XI, WI, true, 2, 2, KW>(p, p.reg[0], wg, smem);
    } else {
        // the rectangles follow each other in the grid, each with its own XCD-aware order
        int r = 0;
        if constexpr (HALF) {
            while (r + 1 < p.n_reg && (long)blockIdx.x >= p.reg[r + 1].first_block) ++r;
        }
        const GcRegion &g = p.reg[r];
        const long local = (long)blockIdx.x - g.first_block;
        const long wg = (local % kXcds) * g.per_xcd + local / kXcds;
        if (wg >= g.tiles) return;
        if constexpr (HALF) {
            if (g.nr == 2 && g.nh == 2) gc_body<TI, TO, WM, XI, WI, false, 2, 2, KW>(p, g, wg, smem);
            else if (g.nr == 2) gc_body<TI, TO, WM, XI, WI, false, 2, 1>(p, g, wg, smem);
            else if (g.nh == 2) gc_body<TI, TO, WM, XI, WI, false, 1, 2>(p, g, wg, smem);
            else gc_body<TI, TO, WM, XI, WI, false, 1, 1>(p, g, wg, smem);
        } else {
            gc_body<TI, TO, WM, XI, WI, false, 2, 2, KW>(p, g, wg, smem);
        }
    }
}

// Adds the pieces of every left-over tile in the order of the workgroups that computed them
// and finishes it.  A workgroup's range is at most NC chunks long, so it meets at most two
// tiles: slot 2g holds the piece its range begins with, 2g+1 the other one.  A thread owns
// kFixRows accumulator registers of one lane of the tile; a tile takes WM*64/kFixRows workgroups.
static constexpr int kFixRows = 8;

template <typename TO, int WM>
__global__ void __launch_bounds__(kThreads)
gc_fixup_kernel(GcParams p)
{
    constexpr int TF = WM * 32;
    constexpr int BPT = WM * 64 / kFixRows;
    const int lt = blockIdx.x / BPT, r0 = (blockIdx.x % BPT) * kFixRows;
    // chunk u belongs to the last workgroup g with g*U/n_wg <= u; U*n_wg < 2^31 by the host's choice
    const int U = p.rem_units, P = (int)p.n_wg;
    const int g_first = ((lt * p.NC + 1) * P + U - 1) / U - 1;
    const int g_last = ((lt + 1) * p.NC * P + U - 1) / U - 1;
    if (g_first == g_last) return;     // one workgroup had the whole tile and finished it
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lo = lane & 31, hi = lane >> 5;
    float acc[kFixRows];
#pragma unroll
    for (int r = 0; r < kFixRows; ++r) acc[r] = 0.f;
    for (int g = g_first; g <= g_last; ++g) {
        const int g_begin = g * U / P;
        if (g_begin == (g + 1) * U / P) continue;     // fewer chunks than workgroups: empty range
        const int second = g_begin / p.NC == lt ? 0 : 1;
        const float *piece = p.partial + (long)(2 * g + second) * (WM * 64 * kThreads) + r0 * kThreads + tid;
#pragma unroll
        for (int r = 0; r < kFixRows; ++r) acc[r] += piece[r * kThreads];
    }
    int fg, n, u0, v0;
    gc_decode_tile(p, p.reg[0], (long)p.rounds * P + lt, fg, n, u0, v0);
    // register r0 + r of the lane is acc[wm][wn][i] of the convolution kernel
    const int wm = r0 / 64, wn = (r0 / 16) % 4, i0 = r0 % 16;
    const int row = u0 + (2 * wave + (wn >> 1)) * p.d;
    const int col = v0 + (wn & 1) * 32 + lo;
    if (row >= p.Hout || col >= p.Wout) return;
    TO *out = (TO *)p.out;
    // the biases are fetched together before the first store (see gc_epilogue); beyond Fout they read zero
    float bv[kFixRows];
    {
        const BufRsrc rb = buf_rsrc(p.bias, p.bias + (p.bias ? p.Fout : 0));
#pragma unroll
        for (int r = 0; r < kFixRows; ++r) {
            const int i = i0 + r;
            bv[r] = buf_ld(rb, p.bias, (unsigned)(fg * TF + wm * 32 + 8 * (i / 4) + 4 * hi + (i % 4)), 0u);
        }
#pragma unroll
        for (int r = 0; r < kFixRows; ++r) asm volatile("" : "+v"(bv[r]));
    }
#pragma unroll
    for (int r = 0; r < kFixRows; ++r) {
        const int i = i0 + r;
        const int f = fg * TF + wm * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
        if (f < p.Fout) stf(out, (((long)n * p.Fimg + f) * p.Hout + row) * p.Wout + col, act_apply(p.act, acc[r] + bv[r]));
    }
}

static constexpr int kXI = 16;   // input-tile elements per thread per chunk, at most
static constexpr int kXIBig = 24;   // the same for tiles with a large halo (second set of kernels)
static constexpr int kWI = 8;    // weight float4s per thread per chunk, at most

struct GcPlan {
    bool ok, split;      // split: persistent workgroups with split tiles
    bool half;           // some rectangle has tiles of half the height or width
    int TF, WM, Cc, Cpad, NC, rows, cols, chan_stride, xs_floats, n_xi, n_wi, n_fgrp, n_rowtile, n_coltile, nrb, full_cls;
    int XI;              // kXI or kXIBig: which set of kernels
    GcRegion reg[4];
    int n_reg;
    long grid;           // physical workgroups when every workgroup takes one tile
    long tiles, n_wg;
    int rounds, rem_units;
    size_t lds_bytes, wt_bytes, partial_bytes;
};

// rectangle [u_base, u_base + Hr) x [v_base, v_base + Wr) of the output map in tiles of 4*nr rows by 32*nh columns
static GcRegion gc_region(int nr, int nh, int u_base, int v_base, int Hr, int Wr, int N, int n_fgrp, int kh, int kw,
                          int d, int Cc)
{
    GcRegion g{};
    const int th = 4 * nr, tw = 32 * nh;
    g.nr = nr; g.nh = nh; g.u_base = u_base; g.v_base = v_base;
    g.rows = th + kh - 1;
    g.cols = tw + (kw - 1) * d;
    g.chan_stride = g.rows * g.cols;
    g.m_cs = (unsigned)((1ull << 32) / (unsigned)g.chan_stride + 1);
    g.m_cols = (unsigned)((1ull << 32) / (unsigned)g.cols + 1);
    g.n_xi = (Cc * g.chan_stride + kThreads - 1) / kThreads;
    // residue classes of the last row block that start beyond the rectangle hold no output: not enumerated
    const int nrb = (Hr + d * th - 1) / (d * th);
    const int last = Hr - (nrb - 1) * d * th;
    g.n_rowtile = (nrb - 1) * d + (last < d ? last : d);
    g.nrb = nrb;
    g.full_cls = last < d ? last : d;
    g.n_coltile = (Wr + tw - 1) / tw;
    g.tiles = (long)N * g.n_rowtile * g.n_coltile * n_fgrp;
    g.per_xcd = (g.tiles + kXcds - 1) / kXcds;
    return g;
}

// Cin / Fout: channel and output counts of the GEMM (swapped for backward-data); N images of
// Hout x Wout outputs
static GcPlan gc_plan(int N, int Cin, int Fout, int Hout, int Wout, int kh, int kw, int d)
{
    GcPlan g{};
    const long kSlots = 2L * device_cu_count();      // workgroups resident at once: two per CU
    g.WM = Fout > 32 ? 2 : 1;
    g.TF = g.WM * 32;
    g.n_fgrp = (Fout + g.TF - 1) / g.TF;
    g.rows = TH + kh - 1;
    const long cols = (long)TW + (long)(kw - 1) * d;
    const long taps = (long)kh * kw;
    if (cols > 4096 || taps > 1024) return g;
    g.cols = (int)cols;
    g.chan_stride = g.rows * g.cols;
    int best = 0, best_pad = 0;
    // both LDS parts are padded to what 256 threads write in whole rounds
    auto xs_padded = [&](int cc) { return (size_t)((cc * g.chan_stride + kThreads - 1) / kThreads * kThreads); };
    auto w_padded = [&](int cc) { return (size_t)((cc * taps * g.TF + 4 * kThreads - 1) / (4 * kThreads) * (4 * kThreads)); };
    for (int xi : {kXI, kXIBig}) {
        for (int cc = 8; cc >= 2; cc -= 2) {
            if (xs_padded(cc) > (size_t)xi * kThreads || w_padded(cc) > (size_t)4 * kWI * kThreads) continue;
            if (4 * (xs_padded(cc) + w_padded(cc)) > kMaxLds) continue;
            const int pad = (Cin + cc - 1) / cc * cc;
            if (best == 0 || pad < best_pad) { best = cc; best_pad = pad; }
        }
        g.XI = xi;
        if (best != 0) break;
    }
    if (best == 0) return g;
    g.Cc = best;
    g.Cpad = best_pad;
    g.NC = g.Cpad / g.Cc;
    g.xs_floats = (int)xs_padded(g.Cc);
    g.n_xi = g.xs_floats / kThreads;
    g.n_wi = (int)(w_padded(g.Cc) / (4 * kThreads));
    g.lds_bytes = 4 * ((size_t)g.xs_floats + w_padded(g.Cc));
    g.wt_bytes = (4 * (size_t)g.n_fgrp * g.Cpad * taps * g.TF + 255) & ~(size_t)255;
    // residue classes of the last row block that start beyond the map hold no output: not enumerated
    {
        const int nrb = (Hout + d * TH - 1) / (d * TH);
        const int last = Hout - (nrb - 1) * d * TH;
        g.n_rowtile = (nrb - 1) * d + (last < d ? last : d);
        g.nrb = nrb;
        g.full_cls = last < d ? last : d;
    }
    g.n_coltile = (Wout + TW - 1) / TW;
    g.tiles = (long)N * g.n_rowtile * g.n_coltile * g.n_fgrp;
    // Tiles are all equally long, so with T tiles and S resident workgroups the last round of a
    // one-tile-per-workgroup launch leaves S - (T mod S) slots idle.  When that costs more than
    // a few per cent, S persistent workgroups take T/S whole tiles each and share the channel
    // chunks of the remaining T mod S tiles evenly.
    // The same machinery fills the chip when there are fewer tiles than slots (small maps): with no whole
    // round, the S workgroups share the channel chunks of ALL tiles (a share is then shorter than a tile,
    // so it still meets two tiles at most).
    // (NC <= 4096 keeps the 32-bit chunk arithmetic of the kernels exact)
    const bool tail = g.tiles > kSlots && g.tiles < 12 * kSlots && g.tiles % kSlots != 0;
    // (tiles of at least four chunks: a piece costs a 64-128 KB round trip through the workspace, which two
    // chunks of a 3-channel layer do not repay)
    const bool few = g.tiles <= kSlots * 3 / 4 && g.NC >= 4 && g.tiles * g.NC >= kSlots / 2;
    g.split = (tail || few) && g.NC <= 4096;
    if (g.split) {
        g.n_wg = kSlots;
        g.rounds = (int)(g.tiles / g.n_wg);
        g.rem_units = (int)(g.tiles - g.rounds * g.n_wg) * g.NC;
        g.partial_bytes = 4 * (size_t)(2 * g.n_wg) * g.WM * 64 * kThreads;
    } else {
        g.n_wg = g.tiles;
        g.rounds = 0;
        g.rem_units = 0;
        g.partial_bytes = 0;
    }
    // Rectangles.  One tile per workgroup and ordinary halos: where the last strip of rows (columns) would fill
    // its tiles at most half -- at most 4 rows per residue class, at most 32 columns -- it becomes a rectangle of
    // its own with tiles of half the height (width).  The rows before it are whole row blocks of 8*d rows, so every
    // residue class keeps its tiles.
    g.reg[0] = gc_region(2, 2, 0, 0, Hout, Wout, N, g.n_fgrp, kh, kw, d, g.Cc);
    g.n_reg = 1;
    g.half = false;
    if (g.XI == kXI) {
        const int hrem = Hout % (TH * d), wrem = Wout % TW;
        const int h_main = hrem > 0 && hrem <= 4 * d ? Hout - hrem : Hout;
        const int w_main = wrem > 0 && wrem <= 32 ? Wout - wrem : Wout;
        if (h_main < Hout || w_main < Wout) {
            GcRegion reg[4];
            int n_reg = 0;
            double work = 0.;      // in whole tiles
            for (int ri = 0; ri < 2; ++ri) {
                const int u_base = ri ? h_main : 0, hr = ri ? Hout - h_main : h_main;
                for (int ci = 0; ci < 2; ++ci) {
                    const int v_base = ci ? w_main : 0, wr = ci ? Wout - w_main : w_main;
                    if (hr <= 0 || wr <= 0) continue;
                    reg[n_reg] = gc_region(ri ? 1 : 2, ci ? 1 : 2, u_base, v_base, hr, wr, N, g.n_fgrp, kh, kw, d, g.Cc);
                    work += (double)reg[n_reg].tiles * reg[n_reg].nr * reg[n_reg].nh / 4.;
                    ++n_reg;
                }
            }
            // Persistent workgroups balance the tail of the grid exactly; one tile per workgroup with small tiles
            // last balances it nearly as well (the small tiles fill the last round) and does less work.  Take
            // the rectangles when that saves more than the quarter of a round the uneven end may cost.
            const bool tail_split = g.split && g.tiles > kSlots;
            const bool few_split = g.split && !tail_split;
            if (!few_split && (!g.split || work / kSlots + 0.25 < (double)g.tiles / kSlots)) {
                for (int r = 0; r < n_reg; ++r) g.reg[r] = reg[r];
                g.n_reg = n_reg;
                g.half = true;
                if (g.split) {
                    g.split = false;
                    g.n_wg = g.tiles;
                    g.rounds = 0;
                    g.rem_units = 0;
                    g.partial_bytes = 0;
                }
            }
        }
    }
    g.grid = 0;
    for (int r = 0; r < g.n_reg; ++r) {
        g.reg[r].first_block = g.grid;
        g.grid += g.reg[r].per_xcd * kXcds;
    }
    g.ok = true;
    return g;
}

template <typename TI, typename TO>
static void gc_launch(const GcParams &p, const GcPlan &g, hipStream_t st)
{
    const unsigned grid = (unsigned)(g.split ? p.per_xcd * kXcds : g.grid);
    if (g.XI == kXIBig && g.WM == 2 && g.split)
        gemm_conv_kernel<TI, TO, 2, kXIBig, kWI, true, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.XI == kXIBig && g.WM == 2)
        gemm_conv_kernel<TI, TO, 2, kXIBig, kWI, false, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.XI == kXIBig && g.split)
        gemm_conv_kernel<TI, TO, 1, kXIBig, kWI, true, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.XI == kXIBig)
        gemm_conv_kernel<TI, TO, 1, kXIBig, kWI, false, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.WM == 2 && g.split)
        gemm_conv_kernel<TI, TO, 2, kXI, kWI, true, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    // the 64-filter kernels for 4 and 5 taps per row have the row unrolled at compile time (1-2 % faster; every
    // further width costs half a minute of compile time)
#define DSK_GC_KW(KW_)                                                                                                   \
    else if (g.WM == 2 && g.half && p.kw == KW_ && p.kh == KW_)                                                                       \
        gemm_conv_kernel<TI, TO, 2, kXI, kWI, false, true, KW_><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);   \
    else if (g.WM == 2 && p.kw == KW_ && p.kh == KW_)                                                                                \
        gemm_conv_kernel<TI, TO, 2, kXI, kWI, false, false, KW_><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    DSK_GC_KW(3)
    DSK_GC_KW(4)
    DSK_GC_KW(5)
#undef DSK_GC_KW
    // ... and the 32-filter kernel for 5 taps (the first layer, backward-data into 32 channels)
    else if (g.WM == 1 && !g.split && g.half && p.kw == 5 && p.kh == 5)
        gemm_conv_kernel<TI, TO, 1, kXI, kWI, false, true, 5><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.WM == 1 && !g.split && p.kw == 5 && p.kh == 5)
        gemm_conv_kernel<TI, TO, 1, kXI, kWI, false, false, 5><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.WM == 2 && g.half)
        gemm_conv_kernel<TI, TO, 2, kXI, kWI, false, true><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.WM == 2)
        gemm_conv_kernel<TI, TO, 2, kXI, kWI, false, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.split)
        gemm_conv_kernel<TI, TO, 1, kXI, kWI, true, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else if (g.half)
        gemm_conv_kernel<TI, TO, 1, kXI, kWI, false, true><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    else
        gemm_conv_kernel<TI, TO, 1, kXI, kWI, false, false><<<dim3(grid), dim3(kThreads), g.lds_bytes, st>>>(p);
    if (g.split) {
        const unsigned left = (unsigned)(g.rem_units / g.NC);
        if (g.WM == 2)
            gc_fixup_kernel<TO, 2><<<dim3(left * (2 * 64 / kFixRows)), dim3(kThreads), 0, st>>>(p);
        else
            gc_fixup_kernel<TO, 1><<<dim3(left * (64 / kFixRows)), dim3(kThreads), 0, st>>>(p);
    }
}

// One launch for the outputs f0 .. f0+Fout-1 of the Fimg the layer has.
static int gc_run_part(const void *in, void *out, const float *w, const float *bias, int N, int Cin, int Hin, int Win,
                       int Fout, int Hout, int Wout, int kh, int kw, int d, int off, int act, int flip,
                       int K, int C, dsk_dtype tin, dsk_dtype tout, void *ws, hipStream_t st, const ConvShape &s, int f0,
                       int Fimg)
{
    const GcPlan g = gc_plan(N, Cin, Fout, Hout, Wout, kh, kw, d);
    if (!g.ok) return DSK_ESHAPE;
    if ((g.n_wg + kXcds - 1) / kXcds * kXcds > 0x7fffffffL || g.grid > 0x7fffffffL) return DSK_ESHAPE;      // before anything is launched
    const int taps = kh * kw;
    float *wt = (float *)ws;
    {
        const long total = (long)g.n_fgrp * g.Cpad * taps * g.TF;
        gc_weight_prep_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
            w, wt, K, C, taps, g.Cpad, g.TF, g.n_fgrp, flip, tin == DSK_BF16 ? 1 : 0, f0, f0 + Fout);
    }
    GcParams p{};
    p.in = in; p.wt = wt;
    p.out = (char *)out + (size_t)f0 * Hout * Wout * (tout == DSK_BF16 ? 2 : 4);
    p.bias = bias ? bias + f0 : nullptr;
    p.Fimg = Fimg;
    p.partial = g.split ? (float *)((char *)ws + g.wt_bytes) : nullptr;
    p.N = N; p.Cin = Cin; p.Hin = Hin; p.Win = Win; p.Fout = Fout; p.Hout = Hout; p.Wout = Wout;
    p.kh = kh; p.kw = kw; p.d = d; p.off_h = off ? (kh - 1) * d : 0; p.off_w = off ? (kw - 1) * d : 0;
    p.act = act;
    p.Cpad = g.Cpad; p.Cc = g.Cc; p.NC = g.NC;
    p.xs_floats = g.xs_floats; p.n_wi = g.n_wi; p.n_fgrp = g.n_fgrp;
    for (int r = 0; r < g.n_reg; ++r) p.reg[r] = g.reg[r];
    p.n_reg = g.n_reg;
    p.tiles = g.tiles; p.rounds = g.rounds; p.rem_units = g.rem_units; p.n_wg = g.n_wg;
    p.per_xcd = (p.n_wg + kXcds - 1) / kXcds;
    if (p.per_xcd * kXcds > 0x7fffffffL) return DSK_ESHAPE;
    p.gsize = s.gsize; p.gjump = s.gjump; p.bgroup = s.bgroup; p.bskip = s.bskip;
    p.in_bstride = (long)(s.gsize ? s.gsize : Cin) * Hin * Win;
    p.in_extent = s.in_extent ? s.in_extent : (long)N * Cin * Hin * Win;
    if (tin == DSK_F32 && tout == DSK_F32) gc_launch<float, float>(p, g, st);
    else if (tin == DSK_F32 && tout == DSK_BF16) gc_launch<float, bf16>(p, g, st);
    else if (tin == DSK_BF16 && tout == DSK_BF16) gc_launch<bf16, bf16>(p, g, st);
    else gc_launch<bf16, float>(p, g, st);
    return check_launch();
}

// A layer whose filter count leaves at most 32 for the last 64-filter group would compute that group at half use:
// the whole groups and the last 32 filters then run as two launches, the second with 32-filter tiles.
static int gc_tail(int Fout) { return Fout > 64 && (Fout - 1) % 64 < 32 ? (Fout - 1) % 64 + 1 : 0; }

static size_t gc_ws_bytes(int N, int Cin, int Fout, int Hout, int Wout, int kh, int kw, int d)
{
    const int tail = gc_tail(Fout);
    if (tail) {
        const GcPlan a = gc_plan(N, Cin, Fout - tail, Hout, Wout, kh, kw, d), b = gc_plan(N, Cin, tail, Hout, Wout, kh, kw, d);
        if (a.ok && b.ok) {
            const size_t wa = a.wt_bytes + a.partial_bytes, wb = b.wt_bytes + b.partial_bytes;
            return wa > wb ? wa : wb;
        }
    }
    const GcPlan g = gc_plan(N, Cin, Fout, Hout, Wout, kh, kw, d);
    return g.ok ? g.wt_bytes + g.partial_bytes : 0;
}

static int gc_run(const void *in, void *out, const float *w, const float *bias, int N, int Cin, int Hin, int Win,
                  int Fout, int Hout, int Wout, int kh, int kw, int d, int off, int act, int flip,
                  int K, int C, dsk_dtype tin, dsk_dtype tout, void *ws, hipStream_t st, const ConvShape &s)
{
    const int tail = gc_tail(Fout);
    if (tail && gc_plan(N, Cin, Fout - tail, Hout, Wout, kh, kw, d).ok && gc_plan(N, Cin, tail, Hout, Wout, kh, kw, d).ok) {
        const int rc = gc_run_part(in, out, w, bias, N, Cin, Hin, Win, Fout - tail, Hout, Wout, kh, kw, d, off, act, flip, K, C,
                                   tin, tout, ws, st, s, 0, Fout);
        if (rc != DSK_OK) return rc;
        return gc_run_part(in, out, w, bias, N, Cin, Hin, Win, tail, Hout, Wout, kh, kw, d, off, act, flip, K, C, tin, tout,
                           ws, st, s, Fout - tail, Fout);
    }
    return gc_run_part(in, out, w, bias, N, Cin, Hin, Win, Fout, Hout, Wout, kh, kw, d, off, act, flip, K, C, tin, tout, ws, st,
                       s, 0, Fout);
}

// ============================================================================
// 1x1 kernels (the last fully connected layers): out[n][f][q] = epi( sum_c wt[c][f] * in[n][c][q] )
// over the flat pixel index q.  Few filters or few channels make these layers HBM-bound, so
// nothing is staged: a wave owns 128 consecutive pixels and reads both MFMA operands straight
// from global memory -- B (lane = pixel, 128 B per half wave and load) and A (lane = filter,
// from the small re-laid-out weight matrix, which stays in the caches) -- eight channels ahead
// of the matrix cores.  No LDS, no barriers; the waves are independent.
// ============================================================================
static constexpr int kPwCh = 8;     // channels per batch of loads (4 MFMA k-steps)

struct PwParams {
    const void *in;
    void *out;
    const float *wt;     // [n_fgrp][Cpad][TF], zero padded (Cpad a multiple of kPwCh)
    const float *bias;   // may be null
    int N, Cin, Fout, act, Cpad, n_fgrp;
    long HW;             // pixels per plane, < 2^28
    long n_wave;         // N * ceil(HW / (32 NB))
    // GATE (backward-data followed by the non-linearity backward of the layer below, Sec. 4.1):
    const void *gate;    // that layer's stored output, same shape and type as `out` (unused for gact = none)
    float *part;         // [n_wave][Cst]: per-wave sums of the stored values, for that layer's bias gradient
    int gact, Cst;       // Cst = n_fgrp * TF
};

// Sum of 2H values per lane over the lanes that differ in `bit`: the lane with the bit clear keeps the
// sums of the first H values, the other one those of the last H (each sends the half it gives up).
template <int H>
__device__ inline void pw_fold(float *v, bool up, int bit)
{
#pragma unroll
    for (int j = 0; j < H; ++j) {
        const float send = up ? v[j] : v[j + H], keep = up ? v[j + H] : v[j];
        v[j] = keep + __shfl_xor(send, bit);
    }
}

template <typename TI, typename TO, int WM, bool GATE, int NB>
__global__ void __launch_bounds__(kThreads, 2)
pw_conv_kernel(PwParams p)
{
    constexpr int TF = WM * 32, KS = kPwCh / 2;
    const int lane = threadIdx.x & 63, lo = lane & 31, hi = lane >> 5;
    const long wv = (long)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wv >= p.n_wave) return;
    const long per_img = (p.HW + 32 * NB - 1) / (32 * NB);
    const int n = (int)(wv / per_img);
    const unsigned q0 = (unsigned)(wv - n * per_img) * (32u * NB);
    const unsigned HW = (unsigned)p.HW;
    const TI *in_n = (const TI *)p.in + (long)n * p.Cin * p.HW;
    const BufRsrc rin = buf_rsrc(in_n, in_n + (long)p.Cin * p.HW);
    // this lane's pixel of each of the four 32-pixel blocks; pixels beyond the plane read pixel 0
    unsigned qoff[NB];
#pragma unroll
    for (int wn = 0; wn < NB; ++wn) {
        const unsigned q = q0 + 32u * wn + lo;
        qoff[wn] = q < HW ? q : 0u;
    }
    const int NC = p.Cpad / kPwCh;
    for (int fg = 0; fg < p.n_fgrp; ++fg) {
        const float *wg = p.wt + (long)fg * p.Cpad * TF;
        const BufRsrc rw = buf_rsrc(wg, wg + (long)p.Cpad * TF);
        f32x16 acc[WM][NB];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm)
#pragma unroll
            for (int wn = 0; wn < NB; ++wn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[wm][wn][i] = 0.f;
        float a_cur[KS][WM], b_cur[KS][NB], a_nxt[KS][WM], b_nxt[KS][NB];
        // channels at or beyond Cin meet zero weights; they are read from the last channel
        auto fetch = [&](int c0, float (&a)[KS][WM], float (&b)[KS][NB]) __attribute__((always_inline)) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int c = c0 + 2 * s;                      // lanes 32..63 take c + 1
                const unsigned ce = (unsigned)(c < p.Cin ? c : p.Cin - 1), co = (unsigned)(c + 1 < p.Cin ? c + 1 : p.Cin - 1);
#pragma unroll
                for (int wm = 0; wm < WM; ++wm) a[s][wm] = buf_ld(rw, wg, (unsigned)(hi * TF + wm * 32 + lo), (unsigned)c * TF);
#pragma unroll
                for (int wn = 0; wn < NB; ++wn) b[s][wn] = buf_ld(rin, in_n, qoff[wn] + (hi ? co : ce) * HW, 0u);
            }
        };
        fetch(0, a_cur, b_cur);
        for (int ch = 0; ch < NC; ++ch) {
            // the next batch (the last one is fetched twice: a load under a condition would be waited for at once)
            fetch((ch + 1 < NC ? ch + 1 : ch) * kPwCh, a_nxt, b_nxt);
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                    for (int wn = 0; wn < NB; ++wn)
                        acc[wm][wn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[s][wm], b_cur[s][wn], acc[wm][wn], 0, 0, 0);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int wm = 0; wm < WM; ++wm) a_cur[s][wm] = a_nxt[s][wm];
#pragma unroll
                for (int wn = 0; wn < NB; ++wn) b_cur[s][wn] = b_nxt[s][wn];
            }
        }
        // bias, non-linearity, store (register i of a lane: filter 8*(i/4) + i%4 + 4*hi of its block)
        TO *out_n = (TO *)p.out + ((long)n * p.Fout + (long)fg * TF) * p.HW;
        const int f_left = p.Fout - fg * TF;
        if constexpr (GATE) {
            // out = acc * act'(gate), and the sum of what is stored over this wave's 128 pixels, per filter
            const TO *y_n = (const TO *)p.gate + ((long)n * p.Fout + (long)fg * TF) * p.HW;
            const BufRsrc ry = buf_rsrc(y_n, y_n + (p.gact != DSK_ACT_NONE ? (long)f_left * p.HW : 0));   // filters beyond the last read 0
            float sum[WM * 16];
#pragma unroll
            for (int i = 0; i < WM * 16; ++i) sum[i] = 0.f;
#pragma unroll
            for (int wn = 0; wn < NB; ++wn) {
                const unsigned q = q0 + 32u * wn + lo;
                float yv[WM][16];
                if (p.gact != DSK_ACT_NONE) {
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            yv[wm][i] = buf_ld(ry, y_n, qoff[wn] + (hi ? 4u * HW : 0u), (unsigned)(wm * 32 + 8 * (i / 4) + (i % 4)) * HW);
                }
                TO *o = out_n + q + (hi ? 4 * p.HW : 0);
#pragma unroll
                for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int fl = wm * 32 + 8 * (i / 4) + (i % 4);
                        float g = acc[wm][wn][i];      // zero for filters beyond the last (zero weights)
                        if (p.gact == DSK_ACT_RELU) g = yv[wm][i] > 0.f ? g : 0.f;
                        else if (p.gact == DSK_ACT_TANH) g *= 1.f - yv[wm][i] * yv[wm][i];
                        g = round_w<TO>(g);            // the sum is over what the weight gradient will read
                        if (q < HW) {
                            if (fl + 4 * hi < f_left) stf(o, (long)fl * p.HW, g);
                            sum[wm * 16 + i] += g;
                        }
                    }
            }
            // over the 32 pixels of a half wave: lane lo ends with the sum of register lo (WM = 1: lo / 2)
            int idx;
            if constexpr (WM == 2) {
                pw_fold<16>(sum, lo & 16, 16); pw_fold<8>(sum, lo & 8, 8); pw_fold<4>(sum, lo & 4, 4);
                pw_fold<2>(sum, lo & 2, 2); pw_fold<1>(sum, lo & 1, 1);
                idx = lo;
            } else {
                pw_fold<8>(sum, lo & 16, 16); pw_fold<4>(sum, lo & 8, 8); pw_fold<2>(sum, lo & 4, 4);
                pw_fold<1>(sum, lo & 2, 2);
                sum[0] += __shfl_xor(sum[0], 1);
                idx = lo >> 1;
            }
            const int i = idx & 15;
            if (WM == 2 || (lo & 1) == 0)
                p.part[wv * p.Cst + fg * TF + (idx >> 4) * 32 + 8 * (i / 4) + (i % 4) + 4 * hi] = sum[0];
            continue;
        }
        // this lane's biases, fetched together before the first store (see gc_epilogue)
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
        for (int wn = 0; wn < NB; ++wn) {
            const unsigned q = q0 + 32u * wn + lo;
            if (q >= HW) continue;
            TO *o = out_n + q + (hi ? 4 * p.HW : 0);
#pragma unroll
            for (int wm = 0; wm < WM; ++wm)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int fl = wm * 32 + 8 * (i / 4) + (i % 4);
                    if (fl + 4 * hi < f_left) stf(o, (long)fl * p.HW, act_apply(p.act, acc[wm][wn][i] + bv[wm][i]));
                }
        }
    }
}

struct PwPlan {
    bool ok;
    int WM, NB, TF, n_fgrp, Cpad;      // NB: 32-pixel blocks per wave
    size_t wt_bytes;
};

static PwPlan pw_plan(int Cin, int Fout, long HW, int kh, int kw, bool gated = false)
{
    PwPlan g{};
    if (kh != 1 || kw != 1 || HW >= (1L << 28) || (long)Cin * HW >= (1L << 30)) return g;
    // the gated form is bound by the latency of its loads: 32-filter tiles need fewer registers, so three waves
    // per SIMD instead of two (2.86 -> 2.63 ms on a 33 -> 256 layer over 4 x 1024 x 1024 pixels; 64-pixel waves
    // on top of that lose again on bf16 maps, whose rows of 32 pixels are only 64 bytes)
    g.WM = Fout > 32 && !gated ? 2 : 1;
    g.NB = 4;
    g.TF = g.WM * 32;
    g.n_fgrp = (Fout + g.TF - 1) / g.TF;
    g.Cpad = (Cin + kPwCh - 1) / kPwCh * kPwCh;
    g.wt_bytes = (4 * (size_t)g.n_fgrp * g.Cpad * g.TF + 255) & ~(size_t)255;
    g.ok = true;
    return g;
}

template <typename TI, typename TO, bool GATE = false>
static void pw_launch(const PwParams &p, int WM, hipStream_t st)
{
    const unsigned grid = (unsigned)((p.n_wave + 3) / 4);
    if constexpr (GATE) pw_conv_kernel<TI, TO, 1, true, 4><<<dim3(grid), dim3(kThreads), 0, st>>>(p);
    else if (WM == 2) pw_conv_kernel<TI, TO, 2, false, 4><<<dim3(grid), dim3(kThreads), 0, st>>>(p);
    else pw_conv_kernel<TI, TO, 1, false, 4><<<dim3(grid), dim3(kThreads), 0, st>>>(p);
}

// The per-wave sums of the gated kernel, added up in a fixed order: 128 rows per workgroup, then the groups.
// A workgroup takes 64 columns; its four waves take every fourth row of its share (a wave reads 256 contiguous
// bytes of a row) and their sums meet in LDS.
static constexpr int kPwSumRows = 128;

__global__ void __launch_bounds__(kThreads)
pw_gate_sum_kernel(const float *__restrict__ src, float *__restrict__ dst, long n_rows, long rows_per_block, int stride,
                   int n_cols, long dst_stride)
{
    __shared__ float sm[4][64];
    const int c = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int f = blockIdx.y * 64 + c;
    const long r0 = (long)blockIdx.x * rows_per_block, r1 = r0 + rows_per_block < n_rows ? r0 + rows_per_block : n_rows;
    float acc = 0.f;
    if (f < n_cols)
        for (long r = r0 + w; r < r1; r += 4) acc += src[r * stride + f];
    sm[w][c] = acc;
    __syncthreads();
    if (w == 0 && f < n_cols) dst[(long)blockIdx.x * dst_stride + f] = (sm[0][c] + sm[1][c]) + (sm[2][c] + sm[3][c]);
}

// workspace of the gated call: weights | per-wave sums | per-group sums
struct PwGatePlan {
    bool ok;
    PwPlan g;
    long n_wave;
    int n_grp, Cst;
    size_t part_off, part2_off, bytes;
};

static PwGatePlan pw_gate_plan(int N, int Cin, int Fout, long HW, int kh, int kw)
{
    PwGatePlan q{};
    q.g = pw_plan(Cin, Fout, HW, kh, kw, true);
    if (!q.g.ok) return q;
    q.n_wave = (long)N * ((HW + 32 * q.g.NB - 1) / (32 * q.g.NB));
    if ((q.n_wave + 3) / 4 > 0x7fffffffL) return q;
    const long grp = (q.n_wave + kPwSumRows - 1) / kPwSumRows;
    if (grp > 0x7fffffffL) return q;
    q.n_grp = (int)grp;
    q.Cst = q.g.n_fgrp * q.g.TF;
    q.part_off = q.g.wt_bytes;
    q.part2_off = q.part_off + ((4 * (size_t)q.n_wave * q.Cst + 255) & ~(size_t)255);
    q.bytes = q.part2_off + ((4 * (size_t)q.n_grp * q.Cst + 255) & ~(size_t)255);
    q.ok = true;
    return q;
}

// K, C: dimensions of w; flip = 1 for backward-data (GEMM channels = filters of w)
// db != null: the gated form (tin == tout): out = (W^T in) * gact'(gate), db = sums of out per plane
static int pw_run(const void *in, void *out, const float *w, const float *bias, int N, int Cin, int Fout, long HW,
                  int act, int flip, int K, int C, dsk_dtype tin, dsk_dtype tout, void *ws, hipStream_t st,
                  const void *gate = nullptr, float *db = nullptr, int gact = DSK_ACT_NONE)
{
    const PwPlan g = pw_plan(Cin, Fout, HW, 1, 1, db != nullptr);
    if (!g.ok) return DSK_ESHAPE;
    const PwGatePlan gp = db ? pw_gate_plan(N, Cin, Fout, HW, 1, 1) : PwGatePlan{};
    if (db && (!gp.ok || tin != tout)) return DSK_ESHAPE;
    const long n_wave = (long)N * ((HW + 32 * g.NB - 1) / (32 * g.NB));
    if ((n_wave + 3) / 4 > 0x7fffffffL) return DSK_ESHAPE;      // before anything is launched
    float *wt = (float *)ws;
    const long total = (long)g.n_fgrp * g.Cpad * g.TF;
    gc_weight_prep_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
        w, wt, K, C, 1, g.Cpad, g.TF, g.n_fgrp, flip, tin == DSK_BF16 ? 1 : 0, 0, Fout);
    PwParams p{};
    p.in = in; p.out = out; p.wt = wt; p.bias = bias;
    p.N = N; p.Cin = Cin; p.Fout = Fout; p.act = act; p.Cpad = g.Cpad; p.n_fgrp = g.n_fgrp;
    p.HW = HW; p.n_wave = n_wave;
    if (db) {
        p.gate = gate; p.gact = gact; p.Cst = gp.Cst;
        p.part = (float *)((char *)ws + gp.part_off);
        float *part2 = (float *)((char *)ws + gp.part2_off);
        if (tin == DSK_F32) pw_launch<float, float, true>(p, g.WM, st);
        else pw_launch<bf16, bf16, true>(p, g.WM, st);
        pw_gate_sum_kernel<<<dim3((unsigned)gp.n_grp, (unsigned)((gp.Cst + 63) / 64)), dim3(kThreads), 0, st>>>(
            p.part, part2, gp.n_wave, kPwSumRows, gp.Cst, gp.Cst, gp.Cst);
        pw_gate_sum_kernel<<<dim3(1u, (unsigned)((Fout + 63) / 64)), dim3(kThreads), 0, st>>>(
            part2, db, gp.n_grp, gp.n_grp, gp.Cst, Fout, 0);
        return check_launch();
    }
    if (tin == DSK_F32 && tout == DSK_F32) pw_launch<float, float>(p, g.WM, st);
    else if (tin == DSK_F32 && tout == DSK_BF16) pw_launch<float, bf16>(p, g.WM, st);
    else if (tin == DSK_BF16 && tout == DSK_BF16) pw_launch<bf16, bf16>(p, g.WM, st);
    else pw_launch<bf16, float>(p, g.WM, st);
    return check_launch();
}

// ============================================================================
// backward-weight: dw[f][c][a][b] = sum_{n,u,v} dy[n][f][u][v] * x[n][c][u+a*d][v+b*d]
// One workgroup owns a 32-filter x 32-channel block of dw for ALL taps and walks over
// a share of the pixel tiles (split-K); the four waves divide the taps.  Partial
// blocks go to the workspace and are summed in a fixed order by a second kernel.
// ============================================================================
static constexpr int PH = 4;    // pixel-tile rows (one residue class mod d)
static constexpr int PW = 32;   // pixel-tile columns
static constexpr int DY_STRIDE = PH * PW + 2;   // the larger of the two pitches of the dy tile (see the kernel)

// loads for the tiles of the weight gradient
__device__ inline float bw_ld(BufRsrc r, const float *p, unsigned lane_off, unsigned uniform_off) { return buf_ld(r, p, lane_off, uniform_off); }
__device__ inline float bw_ld(BufRsrc r, const bf16 *p, unsigned lane_off, unsigned uniform_off) { return buf_ld(r, p, lane_off, uniform_off); }
__device__ inline float bw_ld(const float *p, long i) { return p[i]; }
__device__ inline float bw_ld(const bf16 *p, long i) { return bf16_to_f32(p[i]); }

struct BwParams {
    const void *x, *dy;
    float *part;         // [split][taps][Kp][Cp]
    int N, C, H, W, K, Ho, Wo, kh, kw, d;
    int n_pass;          // > 1: a wide kernel is taken one tap column at a time; pass b reads x b*d columns to the right
    long pass_stride;    // floats of `part` per pass
    int Kp, Cp;          // padded to 32
    int xrows, xcols, xstride;   // x tile: PH+kh-1 by PW+(kw-1)*d, channel stride odd
    int n_rowtile, n_coltile;    // pixel tiles per image
    long n_ptile;        // N * n_rowtile * n_coltile
    int S;               // split count
    int n_fblk, n_cblk;
    int bgroup, bskip;   // image n of x sits at slot n + n / bgroup * bskip (video layers; see ConvShape)
    long x_extent;       // readable elements of x
    // A workgroup's next pixel tile is S tiles further on: S = (step_n * n_rowtile + step_rt) * n_coltile + step_ct,
    // so that the tile's (image, row tile, column tile) follow by additions with carry instead of three divisions
    // per tile, and d_magic = floor(2^32 / d) + 1 turns rt / d into one multiplication (rt, d < 2^16; unused for d = 1).
    int step_ct, step_rt, step_n;
    unsigned d_magic;
};

// TPW: accumulator tiles (taps) per wave; XR: rows of the x tile, at most.
// ROWSPLIT = false: the four waves divide the taps (wave, wave+4, ...) and each walks over the
//   whole pixel tile.  ROWSPLIT = true (few taps): every wave takes ALL taps but only row
//   `wave` of the pixel tile; its block is then one more partial sum for the reduce kernel.
// PREFETCH: fetch the next pixel tile into registers while the matrix cores work on the
//   current one (needs the registers); otherwise the loads of a tile are issued together
//   right before it is staged and a second resident workgroup covers their latency.
// PACKB (layers with at most four input channels, e.g. the image): the 32 columns of the B
//   operand are (channel, tap column b) pairs instead of 32 channels, so the accumulator
//   tiles are indexed by the tap ROW only and a 5x5x3 kernel costs 5 MFMA columns of which
//   15/32 are useful instead of 25 of which 3/32 are.
// FB = 2 (3x3 kernels): the workgroup owns TWO 32-filter blocks; waves 0/2 take the first
//   and waves 1/3 the second, and the two waves of a block divide the taps.  The x tile is then
//   staged once per 64 filters, and a staged tile feeds 2.2 times as many matrix instructions
//   as when every wave takes all nine taps of one tile row.
// SHARED (4*(TPW-1) + 1 taps, e.g. 5x5): divided tap by tap, one wave would have TPW taps and the others
//   TPW-1, and all would wait for the one (25 taps: 28 taps' time).  The last tap is therefore shared:
//   every wave takes TPW-1 whole taps and tile row `wave` of the last one, and the four partial tiles of
//   that tap are added through LDS, in wave order, when the workgroup is done.  With FB = 2 (nine taps for the
//   two waves of a block): four whole taps each and two tile rows of the ninth.
template <typename TI, int TPW, int XR, bool ROWSPLIT, bool PREFETCH, bool PACKB = false, int FB = 1, bool SHARED = false>
__global__ void __launch_bounds__(kThreads, (TPW <= 9 ? 2 : 1))
conv_bwd_weight_mfma_kernel(BwParams p)
{
    extern __shared__ __align__(16) float smem[];
    // Instances that stage quads (see below) keep both tiles at pitches of twice an odd number of words -- conflict-free
    // reads with lanes = filters or channels, rows 8-byte aligned; the others at odd pitches (measured: half a percent
    // faster for them).  The host chooses the channel pitch of the x tile by the same rule.
    constexpr bool QUAD = PREFETCH && !PACKB && XR >= 8 && sizeof(TI) == 4;
    constexpr int DYS = QUAD ? PH * PW + 2 : PH * PW + 1;
    float *dys = smem;                       // [32 * FB filters][DYS]
    float *xs = smem + FB * 32 * DYS;        // [32 channels][xstride]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lo = lane & 31, hi = lane >> 5;
    const int taps = PACKB ? p.kh : p.kh * p.kw;     // accumulator tiles per block
    constexpr int NCI = PACKB ? 1 : 8;              // channels of the x tile each wave stages

    // All (filter block, channel block) workgroups of one pixel share are neighbours in the
    // logical order and, through the XCD-aware mapping, run on the same XCD at the same time:
    // the x tiles are then fetched from HBM once, not once per filter block (and dy likewise).
    // The tap-column passes of one pixel share are neighbours too: their x tiles overlap.
    const int nblk = p.n_fblk * p.n_cblk * p.S * p.n_pass;
    const int per_xcd = (nblk + kXcds - 1) / kXcds;
    int b = (int)(blockIdx.x % kXcds) * per_xcd + (int)(blockIdx.x / kXcds);
    if (b >= nblk) return;
    const int fb = b % p.n_fblk; b /= p.n_fblk;      // n_fblk counts groups of FB filter blocks
    const int cb = b % p.n_cblk; b /= p.n_cblk;
    const int pass = b % p.n_pass;
    const int s = b / p.n_pass;
    const int col_shift = pass * p.d;
    const int f_base = fb * 32 * FB;
    const int my_fb = FB == 2 ? wave & 1 : 0;                                   // this wave's block of the group
    const int tap0 = FB == 2 ? wave >> 1 : wave, tap_step = FB == 2 ? 2 : 4;    // its taps: tap0, tap0 + tap_step, ...

    const TI *x = (const TI *)p.x;
    const TI *dy = (const TI *)p.dy;

    // LDS offset of each of this wave's taps; a slot beyond the last tap repeats tap 0 (its
    // products are never written out), which keeps the inner loop branch-free
    int boff[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        int tap = ROWSPLIT ? t : tap0 + tap_step * t;
        tap = tap < taps ? tap : 0;
        if (SHARED && t == TPW - 1) tap = taps - 1;
        const int a = PACKB ? tap : tap / p.kw;
        boff[t] = a * p.xcols + (PACKB ? 0 : (tap - a * p.kw) * p.d);
    }
    // per-lane part of the B address: the lane's channel, and with PACKB also its tap column
    int blane = lo * p.xstride;
    if (PACKB) {
        const int j = lo < p.C * p.kw ? lo : 0;      // lanes beyond the last pair repeat pair 0
        blane = (j / p.kw) * p.xstride + (j % p.kw) * p.d;
    }

    f32x16 acc[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    float dr[16 * FB];       // dy tile share: (filter, row) segments wave*2+hi+8i, column lo
    float xr[NCI][XR];       // x tile share: channels wave+4*ci, rows r, column lane

    // Every tile starts inside both maps (the host enumerates only such tiles), so the tile's
    // base is always a valid address: loads that fall outside the maps are redirected there and
    // replaced by zero when the registers are written to LDS.  Nothing depends on a loaded
    // value before that point, so all loads of a tile are in flight together, and the address
    // is a wave-uniform base plus one per-lane offset shared by all loads of the tile.
    const unsigned HoWo = (unsigned)(p.Ho * p.Wo), dWo = (unsigned)(p.d * p.Wo);
    const unsigned HW = (unsigned)(p.H * p.W), dW = (unsigned)(p.d * p.W);
    const int nf_valid = p.K - f_base, nc_valid = p.C - cb * 32;
    const bool full_blocks = !PACKB && nf_valid >= 32 * FB && nc_valid >= 32;
    const TI *dy_end = dy + (long)p.N * p.K * HoWo, *x_end = x + p.x_extent;
    int st_nr_dy = 0, st_nr_x = 0;             // rows of the staged tile that exist
    bool st_dcol_ok = false, st_col_ok = false; // this lane's column exists
    bool st_full = false;                       // every row, filter and channel of the staged tile exists (uniform)
    // QUAD (full tiles of the fp32 kernels that prefetch; x tiles a multiple of four columns wide and at most eight
    // rows high): a lane loads FOUR neighbouring columns with one 16-byte access.  The vector memory path spends as
    // long on a wave's 4-byte loads as on its 16-byte ones, and the ~72 dword loads per thread and tile cost the
    // kernel an eighth of its time (measured by leaving them out), wherever in the tile they were issued.
    // dy: a wave's load covers two filters (lanes 0-31 / 32-63) x 4 rows x 8 column groups; filter wave*8*FB + 2*i +
    // lane/32.  x: channel wave + 4*ci, items (row, column group) lane and lane + 64 of the xrows * xcols/4.
    // (the kernels that do not prefetch -- 5 x 5 layers -- lose 4 % with it)
    const bool quad = QUAD && p.xcols % 4 == 0 && p.xrows * (p.xcols / 4) <= 128;      // (uniform)
    const int qd_f = lane >> 5, qd_r = (lane & 31) >> 3, qd_g = lane & 7;
    const int qG = p.xcols / 4 > 0 ? p.xcols / 4 : 1;
    const int qx_r0 = lane / qG, qx_g0 = lane - qx_r0 * qG, qx_r1 = (lane + 64) / qG, qx_g1 = lane + 64 - qx_r1 * qG;
    const bool qx_ok0 = lane < p.xrows * qG, qx_ok1 = lane + 64 < p.xrows * qG;
    unsigned st_dmask = 0;                      // QUAD: bit j: column 4*qd_g + j of the staged dy tile lies inside the map
    // STEP (the instances that prefetch, where this arithmetic sits between the barrier and the matrix instructions;
    // the others measured slower with it, the scalar registers it holds being spilled): the coordinates of the next
    // tile to load are kept and stepped instead of being divided out of the tile index.
    constexpr bool STEP = PREFETCH && FB == 1;
    int t_ct = 0, t_rt = 0, t_n = 0;
    if (STEP) { t_ct = s % p.n_coltile; t_rt = (s / p.n_coltile) % p.n_rowtile; t_n = s / p.n_coltile / p.n_rowtile; }
    auto advance = [&]() {
        if (!STEP) return;
        t_ct += p.step_ct;
        const int carry = t_ct >= p.n_coltile ? 1 : 0;
        t_ct -= carry ? p.n_coltile : 0;
        t_rt += p.step_rt + carry;
        const int carry2 = t_rt >= p.n_rowtile ? 1 : 0;
        t_rt -= carry2 ? p.n_rowtile : 0;
        t_n += p.step_n + carry2;
    };
    auto load_tile = [&](long pt) {
        int ct = t_ct, rt = t_rt, n = t_n, rq;
        if constexpr (STEP) {
            rq = p.d == 1 ? rt : (int)__umulhi((unsigned)rt, p.d_magic);      // rt / d
        } else {
            ct = (int)(pt % p.n_coltile);
            rt = (int)((pt / p.n_coltile) % p.n_rowtile);
            n = (int)(pt / ((long)p.n_coltile * p.n_rowtile));
            rq = rt / p.d;
        }
        const int u0 = STEP ? rq * p.d * PH + (rt - rq * p.d) : (rt / p.d) * p.d * PH + (rt % p.d);
        const int v0 = ct * PW;
        const TI *dyt = dy + (((long)n * p.K + f_base) * p.Ho + u0) * p.Wo + v0;
        const long xn = p.bgroup ? n + (long)(n / p.bgroup) * p.bskip : (long)n;
        const TI *xt = x + ((xn * p.C + cb * 32) * p.H + u0) * p.W + v0 + col_shift;
        // dy: segment i of this wave is filter f_i, rows r_i (lanes 0-31) and r_i+1 (lanes 32-63)
        st_dcol_ok = v0 + lo < p.Wo;
        st_col_ok = lane < p.xcols && v0 + lane + col_shift < p.W;
        const unsigned xlane_off = st_col_ok ? (unsigned)lane : 0u;
        if constexpr (STEP) {
            // every row of both tiles exists (no division on this path: all but the tiles at the bottom of a map)
            const bool rows_full = u0 + (PH - 1) * p.d < p.Ho && u0 + (p.xrows - 1) * p.d < p.H;
            st_nr_dy = PH;
            st_nr_x = p.xrows;
            if (!rows_full) {
                st_nr_dy = (p.Ho - u0 + p.d - 1) / p.d;       // dy rows u0 + r*d that exist (>= 1)
                st_nr_x = (p.H - u0 + p.d - 1) / p.d;         // x rows u0 + r*d that exist
            }
        } else {
            st_nr_dy = (p.Ho - u0 + p.d - 1) / p.d;
            st_nr_x = (p.H - u0 + p.d - 1) / p.d;
        }
        st_nr_x = st_nr_x < p.xrows ? st_nr_x : p.xrows;
        st_full = full_blocks && st_nr_dy >= PH && st_nr_x == p.xrows;
        if (st_full) {
            // every row, filter and channel of the tile exists (all but the tiles at the bottom
            // of a map): buffer loads with one per-lane offset for the whole tile and a scalar
            // offset per load; only the lane's column may fall outside (read column 0 then)
            const unsigned dlane_off = st_dcol_ok ? (unsigned)hi * dWo + (unsigned)lo : 0u;
            const BufRsrc rd = buf_rsrc(dyt, dy_end);
            if constexpr (QUAD) {
                if (quad) {
                    // columns beyond the map: dy reads what follows in memory (or zero beyond the tensor) and is
                    // masked at the LDS write; x needs no mask (see there)
                    st_dmask = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) st_dmask |= v0 + 4 * qd_g + j < p.Wo ? 1u << j : 0u;
                    const unsigned dq_off = (unsigned)qd_f * HoWo + (unsigned)qd_r * dWo + 4u * qd_g;
#pragma unroll
                    for (int i = 0; i < 4 * FB; ++i) {
                        const f32x4 q = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                            rd, (int)(dq_off * 4u), (int)((unsigned)(wave * 8 * FB + 2 * i) * HoWo * 4u), 0));
#pragma unroll
                        for (int j = 0; j < 4; ++j) dr[4 * i + j] = q[j];
                    }
                    const BufRsrc rxq = buf_rsrc(xt, x_end);
                    const unsigned xo0 = qx_ok0 ? (unsigned)qx_r0 * dW + 4u * qx_g0 : 0u;
                    const unsigned xo1 = qx_ok1 ? (unsigned)qx_r1 * dW + 4u * qx_g1 : 0u;
#pragma unroll
                    for (int ci = 0; ci < NCI; ++ci) {
                        const int so = (int)((unsigned)(wave + 4 * ci) * HW * 4u);
                        const f32x4 a = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rxq, (int)(xo0 * 4u), so, 0));
                        const f32x4 b = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rxq, (int)(xo1 * 4u), so, 0));
#pragma unroll
                        for (int j = 0; j < 4; ++j) { xr[ci][j] = a[j]; xr[ci][4 + j] = b[j]; }
                    }
                    return;
                }
            }
#pragma unroll
            for (int i = 0; i < 16 * FB; ++i) {
                const int seg = wave * 2 + 8 * i;
                dr[i] = bw_ld(rd, dyt, dlane_off, (unsigned)(seg >> 2) * HoWo + (unsigned)(seg & 3) * dWo);
            }
            const BufRsrc rx = buf_rsrc(xt, x_end);
#pragma unroll
            for (int ci = 0; ci < NCI; ++ci) {
#pragma unroll
                for (int r = 0; r < XR; ++r) {
                    const int rr = r < p.xrows ? r : 0;      // rows beyond the tile are not staged
                    xr[ci][r] = bw_ld(rx, xt, xlane_off, (unsigned)(wave + 4 * ci) * HW + (unsigned)rr * dW);
                }
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < 16 * FB; ++i) {
            const int seg = wave * 2 + 8 * i;              // even: the lower half's segment
            const int f = seg >> 2, r = seg & 3;
            const bool ok_s = f < nf_valid && r < st_nr_dy;   // uniform
            const TI *base = ok_s ? dyt + ((unsigned)f * HoWo + (unsigned)r * dWo) : dyt;
            const bool ok = ok_s && st_dcol_ok && r + hi < st_nr_dy;
            dr[i] = bw_ld(base, (long)(ok ? (unsigned)hi * dWo + (unsigned)lo : 0u));
        }
#pragma unroll
        for (int ci = 0; ci < NCI; ++ci) {
            const int c = wave + 4 * ci;
#pragma unroll
            for (int r = 0; r < XR; ++r) {
                const bool ok_s = c < nc_valid && r < st_nr_x;              // uniform
                const TI *base = ok_s ? xt + ((unsigned)c * HW + (unsigned)r * dW) : xt;
                xr[ci][r] = bw_ld(base, (long)xlane_off);
            }
        }
    };

    long pt = s;
    if (PREFETCH && pt < p.n_ptile) { load_tile(pt); advance(); }
    while (pt < p.n_ptile) {
        if (!PREFETCH) load_tile(pt);
        __syncthreads();        // every wave is done with the previous tile
        if (QUAD && st_full && quad) {
#pragma unroll
            for (int i = 0; i < 4 * FB; ++i) {
                float *dst = dys + (wave * 8 * FB + 2 * i + qd_f) * DYS + qd_r * PW + 4 * qd_g;
                // (rows of both tiles begin at even words: two 8-byte writes per quad)
                f32x2 v0 = {(st_dmask >> 0) & 1u ? dr[4 * i] : 0.f, (st_dmask >> 1) & 1u ? dr[4 * i + 1] : 0.f};
                f32x2 v1 = {(st_dmask >> 2) & 1u ? dr[4 * i + 2] : 0.f, (st_dmask >> 3) & 1u ? dr[4 * i + 3] : 0.f};
                *(f32x2 *)dst = v0;
                *(f32x2 *)(dst + 2) = v1;
            }
#pragma unroll
            for (int ci = 0; ci < NCI; ++ci) {
                // no zeroing (see below): an x entry outside the map only meets dy entries outside their map
                if (qx_ok0) {
                    float *d0 = xs + (wave + 4 * ci) * p.xstride + qx_r0 * p.xcols + 4 * qx_g0;
                    *(f32x2 *)d0 = f32x2{xr[ci][0], xr[ci][1]};
                    *(f32x2 *)(d0 + 2) = f32x2{xr[ci][2], xr[ci][3]};
                }
                if (qx_ok1) {
                    float *d1 = xs + (wave + 4 * ci) * p.xstride + qx_r1 * p.xcols + 4 * qx_g1;
                    *(f32x2 *)d1 = f32x2{xr[ci][4], xr[ci][5]};
                    *(f32x2 *)(d1 + 2) = f32x2{xr[ci][6], xr[ci][7]};
                }
            }
        } else {
        if (PREFETCH && st_full) {      // (uniform) only the lane's column may be outside the map: one mask for all entries
#pragma unroll
            for (int i = 0; i < 16 * FB; ++i) {
                const int seg = wave * 2 + hi + 8 * i;
                const float v = st_dcol_ok ? dr[i] : 0.f;
                dys[(seg >> 2) * DYS + (seg & 3) * PW + lo] = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16 * FB; ++i) {
                const int seg = wave * 2 + hi + 8 * i;
                const bool ok = st_dcol_ok && (seg >> 2) < nf_valid && (seg & 3) < st_nr_dy;
                const float v = ok ? dr[i] : 0.f;
                dys[(seg >> 2) * DYS + (seg & 3) * PW + lo] = v;
            }
        }
        if (lane < p.xcols) {
#pragma unroll
            for (int ci = 0; ci < NCI; ++ci)
#pragma unroll
                for (int r = 0; r < XR; ++r)
                    if (r < p.xrows) {
                        // No zeroing here: an x entry outside the map (it was read from the tile's base instead, a
                        // finite value of the map) only ever meets dy entries outside ITS map, which are zeros,
                        // and the columns of channels beyond C are never written out.
                        const float v = xr[ci][r];
                        xs[(wave + 4 * ci) * p.xstride + r * p.xcols + lane] = v;
                    }
        }
        }
        __syncthreads();
        if (PREFETCH && pt + p.S < p.n_ptile) { load_tile(pt + p.S); advance(); }      // in flight while the matrix cores run
        pt += p.S;
        // ---- matrix cores: k index = pixel pair (columns 2q, 2q+1); A = dy (filters), B = x (channels)
        // Steps of two pixel pairs (one two-address LDS read per operand).  The operands of step s+1 are read into
        // a second set of registers BEFORE the matrix instructions of step s are issued: with one set, a read could
        // only be issued after the instructions that use its registers, and its latency would be exposed once per
        // step.  The eight steps of a tile row are unrolled, so that every offset is an immediate.
        const float *ab = dys + (my_fb * 32 + lo) * DYS + hi;
        const float *bb = xs + blane + hi;
        constexpr int NS = PW / 4;      // steps per row
        float A[2][2], B[2][TPW][2];
        auto lds_step = [&](const float *ar, const float *br, int st, int buf) __attribute__((always_inline)) {
            A[buf][0] = ar[4 * st];
            A[buf][1] = ar[4 * st + 2];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                B[buf][t][0] = br[boff[t] + 4 * st];
                B[buf][t][1] = br[boff[t] + 4 * st + 2];
            }
        };
        const int r_first = ROWSPLIT ? wave : 0, r_last = ROWSPLIT ? wave : PH - 1;
        lds_step(ab + r_first * PW, bb + r_first * p.xcols, 0, 0);
        for (int r = r_first; r <= r_last; ++r) {
            const float *ar = ab + r * PW, *br = bb + r * p.xcols;
            const int rn = r < r_last ? r + 1 : r_first;      // (after the last row: read for nothing)
            const float *arn = ab + rn * PW, *brn = bb + rn * p.xcols;
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                if (st + 1 < NS) lds_step(ar, br, st + 1, (st + 1) & 1);
                else lds_step(arn, brn, 0, 0);
                __builtin_amdgcn_sched_barrier(0);      // the scheduler would sink the reads to their uses, one step later
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int t = 0; t < (SHARED ? TPW - 1 : TPW); ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[st & 1][h], B[st & 1][t][h], acc[t], 0, 0, 0);
                if (SHARED && (FB == 2 ? (r >> 1) == (wave >> 1) : r == wave)) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[TPW - 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[st & 1][h], B[st & 1][TPW - 1][h], acc[TPW - 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- partial block out: part[split][tap][f][c]; lane = channel, registers = filters
    const long split = ROWSPLIT ? (long)s * 4 + wave : s;
    float *part = p.part + pass * p.pass_stride + split * p.Kp * p.Cp * taps;
    if constexpr (SHARED) {
        // the partial tiles of the shared tap (four of one block, or two of each of two blocks): through LDS, added
        // in wave order; every wave writes a quarter (half) of the registers of its block's tile
        __syncthreads();      // every wave is done with the last tile
        float *red = smem;    // [wave][register][lane]
#pragma unroll
        for (int i = 0; i < 16; ++i) red[(wave * 16 + i) * 64 + lane] = acc[TPW - 1][i];
        __syncthreads();
        if (FB == 2) {
            if (f_base + my_fb * 32 < p.Kp) {
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) {
                    const int i = 8 * (wave >> 1) + ii;
                    const float v = red[(my_fb * 16 + i) * 64 + lane] + red[((my_fb + 2) * 16 + i) * 64 + lane];
                    const int f = f_base + my_fb * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
                    part[((long)(taps - 1) * p.Kp + f) * p.Cp + cb * 32 + lo] = v;
                }
            }
        } else {
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const int i = 4 * wave + ii;
                const float v = ((red[i * 64 + lane] + red[(16 + i) * 64 + lane]) + red[(32 + i) * 64 + lane]) + red[(48 + i) * 64 + lane];
                const int f = f_base + 8 * wave + 4 * hi + ii;
                part[((long)(taps - 1) * p.Kp + f) * p.Cp + cb * 32 + lo] = v;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < (SHARED ? TPW - 1 : TPW); ++t) {
        const int tap = ROWSPLIT ? t : tap0 + tap_step * t;
        if (tap >= taps || f_base + my_fb * 32 >= p.Kp) continue;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int f = f_base + my_fb * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
            const int c = cb * 32 + lo;
            part[((long)tap * p.Kp + f) * p.Cp + c] = acc[t][i];      // 32 consecutive channels per store
        }
    }
}

// dw[f][c][t] = sum over the S partial blocks, in a fixed order.  A workgroup takes 32
// consecutive outputs in the order the blocks are stored in ([t][f][c], c fastest: coalesced
// reads) and its eight groups of 32 threads take every eighth block each, with four running
// sums so that loads overlap; the 32 partial sums of an output are then added in one order.
static constexpr int kRedOut = 32, kRedGroups = kThreads / kRedOut;

__device__ inline float bw_reduce_sum(const float *__restrict__ src, long stride, int S, bool valid, float *red)
{
    const int j = threadIdx.x % kRedOut, sg = threadIdx.x / kRedOut;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (valid) {
        int s = sg;
        for (; s + 3 * kRedGroups < S; s += 4 * kRedGroups) {
            a0 += src[s * stride];
            a1 += src[(s + kRedGroups) * stride];
            a2 += src[(s + 2 * kRedGroups) * stride];
            a3 += src[(s + 3 * kRedGroups) * stride];
        }
        for (; s < S; s += kRedGroups) a0 += src[s * stride];
    }
    red[sg * kRedOut + j] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    float v = 0.f;
    if (sg == 0)
        for (int q = 0; q < kRedGroups; ++q) v += red[q * kRedOut + j];
    return v;
}

__global__ void __launch_bounds__(kThreads)
bw_reduce_kernel(const float *__restrict__ part, float *__restrict__ dw, int K, int C, int taps, int Kp, int Cp, int S,
                 int taps_dw, int tap_stride, long pass_stride)
{
    // blockIdx.y: tap-column pass of a wide kernel (its blocks start pass_stride floats further on)
    part += blockIdx.y * pass_stride;
    const int tap_first = (int)blockIdx.y;
    __shared__ float red[kThreads];
    const long total = (long)K * C * taps;
    const long idx = (long)blockIdx.x * kRedOut + threadIdx.x % kRedOut;
    const bool valid = idx < total;
    const int c = (int)(idx % C);
    const int f = (int)((idx / C) % K);
    const int t = (int)(idx / ((long)C * K));
    const long o = ((long)t * Kp + f) * Cp + c;
    const float v = bw_reduce_sum(part + (valid ? o : 0), (long)Kp * Cp * taps, S, valid, red);
    // tap t of the blocks is tap tap_first + t*tap_stride of dw's taps_dw
    if (valid && threadIdx.x < kRedOut) dw[((long)f * C + c) * taps_dw + tap_first + t * tap_stride] = v;
}

// The same for blocks whose 32 columns are (channel, tap column) pairs and whose tiles are tap rows.
__global__ void __launch_bounds__(kThreads)
bw_reduce_packb_kernel(const float *__restrict__ part, float *__restrict__ dw, int K, int C, int kh, int kw, int Kp,
                       int S)
{
    __shared__ float red[kThreads];
    const int CB = C * kw;
    const long total = (long)K * CB * kh;
    const long idx = (long)blockIdx.x * kRedOut + threadIdx.x % kRedOut;
    const bool valid = idx < total;
    const int j = (int)(idx % CB);
    const int f = (int)((idx / CB) % K);
    const int a = (int)(idx / ((long)CB * K));
    const long o = ((long)a * Kp + f) * 32 + j;
    const float v = bw_reduce_sum(part + (valid ? o : 0), (long)Kp * 32 * kh, S, valid, red);
    if (valid && threadIdx.x < kRedOut) dw[(((long)f * C + j / kw) * kh + a) * kw + j % kw] = v;
}

// db[f] = sum over n, u, v of dy, in two fixed-order stages: kBiasSplit workgroups per filter
// each reduce a contiguous share of every image's plane, then one thread per filter adds them.
static constexpr int kBiasSplit = 32;

template <typename TI>
__global__ void __launch_bounds__(kThreads)
bias_partial_kernel(const TI *__restrict__ dy, float *__restrict__ part, int N, int K, long plane)
{
    __shared__ float sm[kThreads];
    const int f = blockIdx.x / kBiasSplit, sp = blockIdx.x % kBiasSplit;
    const long share = (plane + kBiasSplit - 1) / kBiasSplit;
    const long lo = sp * share, hi = lo + share < plane ? lo + share : plane;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) {
        const TI *src = dy + ((long)n * K + f) * plane;
        for (long t = lo + threadIdx.x; t < hi; t += kThreads) acc += ldf(src, t);
    }
    sm[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sm[threadIdx.x] += sm[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = sm[0];
}

__global__ void __launch_bounds__(kThreads)
bias_reduce_kernel(const float *__restrict__ part, float *__restrict__ db, int K)
{
    const int f = blockIdx.x * kThreads + threadIdx.x;
    if (f >= K) return;
    float acc = 0.f;
    for (int sp = 0; sp < kBiasSplit; ++sp) acc += part[f * kBiasSplit + sp];
    db[f] = acc;
}

// ============================================================================
// Weight gradient of a 1x1 kernel: dw[f][c] = sum over images and pixels q of dy[f][q] * x[c][q].
// Both maps should come from HBM once: a workgroup owns up to 64 filters x 256 channels of dw
// (16 accumulator tiles, four per wave) and walks over a share of the 32-pixel tiles of the
// flat pixel index; A = dy (lane = filter), B = x (lane = channel), k = pixel pair, both
// transposed through LDS (row pitch 33: conflict-free).  The next tile is fetched into
// registers meanwhile.  Partial blocks [share][Kp][Cp] are summed by bw_reduce_kernel.
// ============================================================================
static constexpr int kPbQ = 32;          // pixels per tile
static constexpr int kPbPitch = kPbQ + 1;

struct PbParams {
    const void *x, *dy;
    float *part;         // [S][Kp][Cp]
    int N, C, K, Kp, Cp, S, n_cg;
    long HW, n_tile;     // pixels per plane; N * ceil(HW / 32)
};

template <typename TI, int FB>
__global__ void __launch_bounds__(kThreads, 2)
pw_bwd_weight_kernel(PbParams p)
{
    __shared__ float dys[FB * 32 * kPbPitch];
    __shared__ float xs[256 * kPbPitch];
    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = blockIdx.x % p.n_cg, s = blockIdx.x / p.n_cg;
    const int c_base = cg * 256;
    const TI *x = (const TI *)p.x, *dy = (const TI *)p.dy;
    const unsigned HW = (unsigned)p.HW;
    const long per_img = (p.HW + kPbQ - 1) / kPbQ;
    const TI *x_end = x + (long)p.N * p.C * p.HW, *dy_end = dy + (long)p.N * p.K * p.HW;

    f32x16 acc[FB][2];
#pragma unroll
    for (int a = 0; a < FB; ++a)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][j][i] = 0.f;

    // staging share of a thread: pixel lo of rows 2*wave + hi + 8*i (x: 32 channel rows, dy: 4*FB filter rows)
    // QUAD (fp32 maps): four neighbouring pixels of row tid/8 + 32*i with one 16-byte load (x: 8 rows, dy: FB rows) --
    // what the staging costs is the number of load instructions, and this is a quarter of them.
    constexpr bool QUAD = sizeof(TI) == 4;
    const int qrow = tid >> 3, qg = tid & 7;
    float xr[32], dr[4 * FB];
    bool st_q_ok = false;
    unsigned st_qmask = 0;      // QUAD: bit j: pixel 4*qg + j of the staged tile exists
    auto load_tile = [&](long t) __attribute__((always_inline)) {
        const int n = (int)(t / per_img);
        const unsigned q0 = (unsigned)(t - n * per_img) * kPbQ;
        st_q_ok = q0 + lo < HW;
        const TI *xn = x + ((long)n * p.C + c_base) * p.HW, *dn = dy + (long)n * p.K * p.HW;
        const BufRsrc rx = buf_rsrc(xn, x_end), rd = buf_rsrc(dn, dy_end);
        if constexpr (QUAD) {
            // rows that do not exist are read from row 0; a quad that reaches past the plane reads what follows in
            // memory (zero past the tensor); both are zeroed at the LDS write
            st_qmask = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) st_qmask |= q0 + 4u * qg + j < HW ? 1u << j : 0u;
            const unsigned pix = st_qmask ? q0 + 4u * qg : 0u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = qrow + 32 * i;
                const unsigned off = c_base + c < p.C ? (unsigned)c * HW + pix : 0u;
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(off * 4u), 0, 0));
#pragma unroll
                for (int j = 0; j < 4; ++j) xr[4 * i + j] = v[j];
            }
#pragma unroll
            for (int i = 0; i < FB; ++i) {
                const int f = qrow + 32 * i;
                const unsigned off = f < p.K ? (unsigned)f * HW + pix : 0u;
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rd, (int)(off * 4u), 0, 0));
#pragma unroll
                for (int j = 0; j < 4; ++j) dr[4 * i + j] = v[j];
            }
            return;
        }
        // rows that do not exist are read from row 0 (a valid address) and zeroed at the LDS write
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int c = 2 * wave + 8 * i;              // lanes 32..63 take c + 1
            const unsigned lane_off = st_q_ok && c_base + c + hi < p.C ? (unsigned)hi * HW + q0 + lo : 0u;
            xr[i] = buf_ld(rx, xn, lane_off, c_base + c < p.C ? (unsigned)c * HW : 0u);
        }
#pragma unroll
        for (int i = 0; i < 4 * FB; ++i) {
            const int f = 2 * wave + 8 * i;
            const unsigned lane_off = st_q_ok && f + hi < p.K ? (unsigned)hi * HW + q0 + lo : 0u;
            dr[i] = buf_ld(rd, dn, lane_off, f < p.K ? (unsigned)f * HW : 0u);
        }
    };

    long t = s;
    if (t < p.n_tile) load_tile(t);
    while (t < p.n_tile) {
        __syncthreads();        // every wave is done with the previous tile
        if constexpr (QUAD) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = qrow + 32 * i;
                const bool row_ok = c_base + c < p.C;
#pragma unroll
                for (int j = 0; j < 4; ++j) xs[c * kPbPitch + 4 * qg + j] = row_ok && ((st_qmask >> j) & 1u) ? xr[4 * i + j] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < FB; ++i) {
                const int f = qrow + 32 * i;
                const bool row_ok = f < p.K;
#pragma unroll
                for (int j = 0; j < 4; ++j) dys[f * kPbPitch + 4 * qg + j] = row_ok && ((st_qmask >> j) & 1u) ? dr[4 * i + j] : 0.f;
            }
        } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int c = 2 * wave + hi + 8 * i;
            xs[c * kPbPitch + lo] = st_q_ok && c_base + c < p.C ? xr[i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 4 * FB; ++i) {
            const int f = 2 * wave + hi + 8 * i;
            dys[f * kPbPitch + lo] = st_q_ok && f < p.K ? dr[i] : 0.f;
        }
        }
        __syncthreads();
        t += p.S;
        // the next tile, or the last one again (a load under a condition would be waited for at once)
        load_tile(t < p.n_tile ? t : t - p.S);
        const float *ab = dys + lo * kPbPitch + hi;
        const float *bb = xs + (wave * 64 + lo) * kPbPitch + hi;
#pragma unroll 4
        for (int q = 0; q < kPbQ / 2; ++q) {
            float A[FB], B[2];
#pragma unroll
            for (int a = 0; a < FB; ++a) A[a] = ab[a * 32 * kPbPitch + 2 * q];
#pragma unroll
            for (int j = 0; j < 2; ++j) B[j] = bb[j * 32 * kPbPitch + 2 * q];
#pragma unroll
            for (int a = 0; a < FB; ++a)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[a][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[a], B[j], acc[a][j], 0, 0, 0);
        }
    }

    float *part = p.part + (long)s * p.Kp * p.Cp;
#pragma unroll
    for (int a = 0; a < FB; ++a)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = c_base + (2 * wave + j) * 32 + lo;
            if (c >= p.Cp) continue;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int f = a * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
                part[(long)f * p.Cp + c] = acc[a][j][i];
            }
        }
}

struct PbPlan {
    bool ok;
    int Kp, Cp, FB, n_cg, S;
    long n_tile;
    size_t part_bytes;
};

static PbPlan pb_plan(const ConvShape &s)
{
    PbPlan b{};
    if (s.kh != 1 || s.kw != 1 || s.K > 64 || (long)s.H * s.W >= (1L << 28)) return b;
    b.Kp = (s.K + 31) / 32 * 32;
    b.Cp = (s.C + 31) / 32 * 32;
    b.FB = b.Kp / 32;
    b.n_cg = (s.C + 255) / 256;
    b.n_tile = (long)s.N * (((long)s.H * s.W + kPbQ - 1) / kPbQ);
    long S = 512 / b.n_cg;
    if (S > b.n_tile / 4) S = b.n_tile / 4;
    if (S < 1) S = 1;
    b.S = (int)S;
    b.part_bytes = 4 * ((size_t)b.S * b.Kp * b.Cp + (size_t)s.K * kBiasSplit);
    b.ok = true;
    return b;
}

struct BwPlan {
    bool ok;
    int Kp, Cp, xrows, xcols, xstride, n_rowtile, n_coltile, S, n_fblk, n_cblk, tpw;
    bool rowsplit, packb;
    bool fb2;            // two filter blocks per workgroup
    bool bf16_cores;     // the kernel of dsk_bww_bf16.hip writes the partial blocks
    int col_passes;      // > 1: one launch per tap column b (a kh x 1 kernel on x shifted by b*d columns)
    int n_part;          // partial blocks the reduce kernel adds up
    long n_ptile;
    size_t lds_bytes, part_bytes;
};

static BwPlan bw_plan_one(const ConvShape &s, bool allow_packb, dsk_dtype in)
{
    BwPlan b{};
    b.col_passes = 1;
    const long taps = (long)s.kh * s.kw;
    if (taps > 52) return b;
    // few input channels: pack (channel, tap column) pairs into the 32 B-operand columns
    b.packb = allow_packb && s.C <= 4 && s.C * s.kw <= 32 && s.kh >= 2 && s.kh <= 7;
    if (in == DSK_BF16 && !b.packb && bww_bf16_shape(s, &b.Kp, &b.Cp, &b.S)) {
        b.bf16_cores = true;
        b.n_fblk = b.Kp / 32;
        b.n_cblk = b.Cp / 32;
        b.n_part = b.S;
        b.part_bytes = 4 * ((size_t)b.n_part * b.Kp * b.Cp * taps + (size_t)s.K * kBiasSplit);
        b.ok = true;
        return b;
    }
    b.fb2 = !b.packb && taps == 9 && s.K > 32;
    b.rowsplit = !b.packb && !b.fb2 && (taps == 1 || taps == 9);
    b.tpw = b.packb ? 2 : b.rowsplit ? (int)taps : b.fb2 ? 5
          : taps <= 4 ? 1 : taps <= 8 ? 2 : taps <= 16 ? 4 : taps <= 28 ? 7 : 13;
    b.Kp = (s.K + 31) / 32 * 32;
    b.Cp = (s.C + 31) / 32 * 32;
    b.n_fblk = b.Kp / 32;
    b.n_cblk = b.Cp / 32;
    b.xrows = PH + s.kh - 1;
    const long xcols = (long)PW + (long)(s.kw - 1) * s.d;
    // one wave-wide load per x-tile row; kernels staging up to 10 rows exist for 2 and 13
    // accumulator tiles per wave and for the packed form, the others stage up to 8
    if (xcols > 64 || s.kh > (b.tpw == 13 || b.tpw == 2 || b.packb ? 7 : 5)) return b;
    if ((long)s.H * s.W >= (1L << 24)) return b;         // 32-channel block offsets stay below 2^29 elements
    b.xcols = (int)xcols;
    // twice an odd number of words per channel: lanes = channels read conflict-free, and rows of tiles a multiple of
    // four columns wide are 8-byte aligned
    {
        const bool quads = in == DSK_F32 && !b.packb && (b.fb2 || b.tpw == 2 || b.tpw == 4 || (b.tpw == 1 && !(b.rowsplit && b.xrows <= 4)));
        b.xstride = quads ? b.xrows * b.xcols + (6 - b.xrows * b.xcols % 4) % 4 : (b.xrows * b.xcols) | 1;
    }
    b.lds_bytes = 4 * ((size_t)32 * DY_STRIDE + (size_t)32 * b.xstride);
    if (b.fb2) {
        const size_t two = 4 * ((size_t)64 * DY_STRIDE + (size_t)32 * b.xstride);
        if (two <= kMaxLdsBw) {
            b.lds_bytes = two;
        } else {      // wide tap spacing: back to one block per workgroup, every wave all nine taps of a row
            b.fb2 = false;
            b.rowsplit = true;
            b.tpw = (int)taps;
        }
    }
    if (b.lds_bytes > kMaxLdsBw) return b;
    // residue classes of the last row block that start beyond the map hold no pixel: skip them
    {
        const int nrb = (s.Ho + s.d * PH - 1) / (s.d * PH);
        const int last = s.Ho - (nrb - 1) * s.d * PH;
        b.n_rowtile = (nrb - 1) * s.d + (last < s.d ? last : s.d);
    }
    b.n_coltile = (s.Wo + PW - 1) / PW;
    b.n_ptile = (long)s.N * b.n_rowtile * b.n_coltile;
    if (b.n_rowtile >= 65536 || s.d >= 65536) return b;      // the kernel divides row-tile indices by d with a 32-bit multiplication
    const long blocks = (long)(b.fb2 ? (b.n_fblk + 1) / 2 : b.n_fblk) * b.n_cblk;
    long S = 2048 / blocks;
    if (S > (blocks == 1 ? 512 : 256)) S = blocks == 1 ? 512 : 256;      // (a single block: enough shares to fill every workgroup slot)
    if (S > b.n_ptile / 4) S = b.n_ptile / 4;
    if (S < 1) S = 1;
    b.S = (int)S;
    b.n_part = b.rowsplit ? 4 * b.S : b.S;
    b.part_bytes = 4 * ((size_t)b.n_part * b.Kp * b.Cp * (b.packb ? s.kh : taps) + (size_t)s.K * kBiasSplit);
    b.ok = true;
    return b;
}

// A kernel whose tap columns are too far apart for one x tile (more than 64 columns wide) is
// taken one tap column at a time: dw[:, :, :, b] is the weight gradient of a kh x 1 kernel on x
// shifted by b*d columns, with the same dy.
static BwPlan bw_plan(const ConvShape &s, dsk_dtype in)
{
    BwPlan b = bw_plan_one(s, true, in);
    if (b.ok || s.kw == 1) return b;
    ConvShape c = s;
    c.kw = 1;                      // Wo stays that of the whole kernel
    b = bw_plan_one(c, false, in);
    b.col_passes = s.kw;
    // all passes run in one launch: each has its own partial blocks
    b.part_bytes = 4 * ((size_t)b.n_part * b.Kp * b.Cp * s.kh * s.kw + (size_t)s.K * kBiasSplit);
    return b;
}

// ============================================================================
// dispatch
// ============================================================================
// a 2-D call: the kernels that know nothing of grouped planes or batch slots may take it
static bool plain_call(const ConvShape &s) { return s.gsize == 0 && s.bgroup == 0; }
// the 1 x 1 weight gradient kernel below computes on the fp32 matrix cores; bf16 maps of even width go to the bf16 ones
static bool pw_bwd_weight_call(const ConvShape &s, dsk_dtype in)
{
    int kp, cp, sp;
    return plain_call(s) && pb_plan(s).ok && !(in == DSK_BF16 && bww_bf16_shape(s, &kp, &cp, &sp));
}

size_t conv_ws_bytes(int which, const ConvShape &s, dsk_dtype in)
{
    // bf16 maps may take either set of kernels: room for both
    if (in == DSK_BF16 && which != DSK_WS_CONV_BWD_WEIGHT && plain_call(s) && conv_bf16_supported(which, s)) {
        const size_t a = conv_bf16_ws_bytes(which, s), b = conv_ws_bytes(which, s, DSK_F32);
        return a > b ? a : b;
    }
    if (which == DSK_WS_CONV_FWD) {
        const PwPlan pw = pw_plan(s.C, s.K, (long)s.H * s.W, s.kh, s.kw);
        if (pw.ok && plain_call(s)) return pw.wt_bytes;
        return gc_ws_bytes(s.N, s.C, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d);
    }
    if (which == DSK_WS_CONV_BWD_DATA) {
        const PwPlan pw = pw_plan(s.K, s.C, (long)s.H * s.W, s.kh, s.kw);
        if (pw.ok && plain_call(s)) return pw.wt_bytes;
        return gc_ws_bytes(s.N, s.K, s.C, s.H, s.W, s.kh, s.kw, s.d);
    }
    if (which == DSK_WS_CONV_BWD_WEIGHT) {
        const PbPlan pb = pb_plan(s);
        if (pw_bwd_weight_call(s, in)) return pb.part_bytes;
        const BwPlan b = bw_plan(s, in);
        return b.ok ? b.part_bytes : 0;
    }
    return 0;
}

bool conv_mfma_supported(int which, const ConvShape &s, dsk_dtype in, dsk_dtype out)
{
    (void)in;
    (void)out;
    // plane offsets are packed into 28 bits, per-image offsets are 32-bit
    if ((long)s.H * s.W >= (1L << 28) || (long)s.C * s.H * s.W >= (1L << 30) ||
        (long)s.K * s.Ho * s.Wo >= (1L << 30))
        return false;
    // grouped planes: a chunk of at most 8 channels may reach into 8 later groups with 32-bit element offsets
    if (s.gsize && (s.gjump < 0 || 8 * (s.gjump + (long)s.H * s.W) >= (1L << 30))) return false;
    if (which == DSK_WS_CONV_FWD)
        return (plain_call(s) && pw_plan(s.C, s.K, (long)s.H * s.W, s.kh, s.kw).ok) || gc_plan(s.N, s.C, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d).ok;
    if (which == DSK_WS_CONV_BWD_DATA)
        return (plain_call(s) && pw_plan(s.K, s.C, (long)s.H * s.W, s.kh, s.kw).ok) || gc_plan(s.N, s.K, s.C, s.H, s.W, s.kh, s.kw, s.d).ok;
    if (which == DSK_WS_CONV_BWD_WEIGHT) return pw_bwd_weight_call(s, in) || bw_plan(s, in).ok;
    return false;
}

int launch_conv_fwd_mfma(const void *x, const float *w, const float *b, void *y, const ConvShape &s,
                         dsk_dtype in, dsk_dtype out, int act, void *ws, hipStream_t st)
{
    if (plain_call(s) && pw_plan(s.C, s.K, (long)s.H * s.W, s.kh, s.kw).ok)
        return pw_run(x, y, w, b, s.N, s.C, s.K, (long)s.H * s.W, act, 0, s.K, s.C, in, out, ws, st);
    return gc_run(x, y, w, b, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo, s.kh, s.kw, s.d, 0, act, 0,
                  s.K, s.C, in, out, ws, st, s);
}

int launch_conv_bwd_data_mfma(const void *dy, const float *w, void *dx, const ConvShape &s,
                              dsk_dtype in, dsk_dtype out, void *ws, hipStream_t st)
{
    if (plain_call(s) && pw_plan(s.K, s.C, (long)s.H * s.W, s.kh, s.kw).ok)
        return pw_run(dy, dx, w, nullptr, s.N, s.K, s.C, (long)s.H * s.W, DSK_ACT_NONE, 1, s.K, s.C, in, out, ws, st);
    return gc_run(dy, dx, w, nullptr, s.N, s.K, s.Ho, s.Wo, s.C, s.H, s.W, s.kh, s.kw, s.d, 1, DSK_ACT_NONE, 1,
                  s.K, s.C, in, out, ws, st, s);
}

// Backward-data with the non-linearity backward and the bias gradient of the layer below in its epilogue:
// 1 x 1 layers on plain 2-D maps of one type (the error map is then written once instead of written, read and rewritten).
bool conv_bwd_data_act_fused(const ConvShape &s, dsk_dtype in, dsk_dtype out)
{
    return in == out && plain_call(s) && conv_mfma_supported(DSK_WS_CONV_BWD_DATA, s, in, out) &&
           pw_gate_plan(s.N, s.K, s.C, (long)s.H * s.W, s.kh, s.kw).ok;
}

size_t conv_bwd_data_act_ws_bytes(const ConvShape &s)
{
    return pw_gate_plan(s.N, s.K, s.C, (long)s.H * s.W, s.kh, s.kw).bytes;
}

int launch_conv_bwd_data_act(const void *dy, const float *w, const void *x, void *dx, float *db, const ConvShape &s,
                             dsk_dtype t, int act, void *ws, hipStream_t st)
{
    return pw_run(dy, dx, w, nullptr, s.N, s.K, s.C, (long)s.H * s.W, DSK_ACT_NONE, 1, s.K, s.C, t, t, ws, st, x, db, act);
}

int launch_conv_bwd_weight_mfma(const void *x, const void *dy, float *dw, float *db, const ConvShape &s,
                                dsk_dtype in, void *ws, hipStream_t st)
{
    if (const PbPlan pb = pb_plan(s); pw_bwd_weight_call(s, in)) {
        PbParams q{};
        q.x = x; q.dy = dy; q.part = (float *)ws;
        q.N = s.N; q.C = s.C; q.K = s.K; q.Kp = pb.Kp; q.Cp = pb.Cp; q.S = pb.S; q.n_cg = pb.n_cg;
        q.HW = (long)s.H * s.W; q.n_tile = pb.n_tile;
        const unsigned grid = (unsigned)(pb.S * pb.n_cg);
        if (in == DSK_F32 && pb.FB == 2) pw_bwd_weight_kernel<float, 2><<<dim3(grid), dim3(kThreads), 0, st>>>(q);
        else if (in == DSK_F32) pw_bwd_weight_kernel<float, 1><<<dim3(grid), dim3(kThreads), 0, st>>>(q);
        else if (pb.FB == 2) pw_bwd_weight_kernel<bf16, 2><<<dim3(grid), dim3(kThreads), 0, st>>>(q);
        else pw_bwd_weight_kernel<bf16, 1><<<dim3(grid), dim3(kThreads), 0, st>>>(q);
        int rc = check_launch();
        if (rc != DSK_OK) return rc;
        const long total = (long)s.K * s.C;
        bw_reduce_kernel<<<dim3((unsigned)((total + kRedOut - 1) / kRedOut)), dim3(kThreads), 0, st>>>(
            (const float *)ws, dw, s.K, s.C, 1, pb.Kp, pb.Cp, pb.S, 1, 1, 0);
        rc = check_launch();
        if (rc != DSK_OK || !db) return rc;
        float *bpart = (float *)ws + (size_t)pb.S * pb.Kp * pb.Cp;
        if (in == DSK_F32)
            bias_partial_kernel<float><<<dim3(s.K * kBiasSplit), dim3(kThreads), 0, st>>>((const float *)dy, bpart, s.N,
                                                                                        s.K, (long)s.Ho * s.Wo);
        else
            bias_partial_kernel<bf16><<<dim3(s.K * kBiasSplit), dim3(kThreads), 0, st>>>((const bf16 *)dy, bpart, s.N,
                                                                                       s.K, (long)s.Ho * s.Wo);
        bias_reduce_kernel<<<dim3((s.K + kThreads - 1) / kThreads), dim3(kThreads), 0, st>>>(bpart, db, s.K);
        return check_launch();
    }
    const BwPlan b = bw_plan(s, in);
    if (!b.ok) return DSK_ESHAPE;
    const int kw_pass = b.col_passes > 1 ? 1 : s.kw;      // tap columns one launch covers
    const int taps = s.kh * kw_pass;
    BwParams p{};
    p.x = x; p.dy = dy; p.part = (float *)ws;
    p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.Ho = s.Ho; p.Wo = s.Wo;
    p.kh = s.kh; p.kw = kw_pass; p.d = s.d;
    p.Kp = b.Kp; p.Cp = b.Cp; p.xrows = b.xrows; p.xcols = b.xcols; p.xstride = b.xstride;
    p.n_rowtile = b.n_rowtile; p.n_coltile = b.n_coltile; p.n_ptile = b.n_ptile; p.S = b.S;
    if (!b.bf16_cores) {      // (that kernel has its own tiles)
        p.step_ct = b.S % b.n_coltile; p.step_rt = (b.S / b.n_coltile) % b.n_rowtile; p.step_n = b.S / b.n_coltile / b.n_rowtile;
    }
    p.d_magic = s.d > 1 ? (unsigned)((1ull << 32) / (unsigned)s.d + 1) : 0u;
    p.n_fblk = b.fb2 ? (b.n_fblk + 1) / 2 : b.n_fblk; p.n_cblk = b.n_cblk;
    p.n_pass = b.col_passes;
    p.bgroup = s.bgroup; p.bskip = s.bskip;
    p.x_extent = s.in_extent ? s.in_extent : (long)s.N * s.C * s.H * s.W;
    p.pass_stride = (long)b.n_part * b.Kp * b.Cp * taps;
    const unsigned grid = (unsigned)(((long)p.n_fblk * b.n_cblk * b.S * b.col_passes + kXcds - 1) / kXcds * kXcds);
#define DSK_BW_LAUNCH(TPW, XR, RS, PF, PB)                                                                 \
    do {                                                                                               \
        if (in == DSK_F32) {                                                                           \
            allow_lds<&conv_bwd_weight_mfma_kernel<float, TPW, XR, RS, PF, PB>>(b.lds_bytes);               \
            conv_bwd_weight_mfma_kernel<float, TPW, XR, RS, PF, PB>                                        \
                <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);                                  \
        } else {                                                                                       \
            allow_lds<&conv_bwd_weight_mfma_kernel<bf16, TPW, XR, RS, PF, PB>>(b.lds_bytes);                \
            conv_bwd_weight_mfma_kernel<bf16, TPW, XR, RS, PF, PB>                                         \
                <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);                                  \
        }                                                                                              \
    } while (0)
#define DSK_BW_LAUNCH_SHARED(TPW, XR)                                                                     \
    do {                                                                                               \
        if (in == DSK_F32) {                                                                           \
            allow_lds<&conv_bwd_weight_mfma_kernel<float, TPW, XR, false, false, false, 1, true>>(b.lds_bytes);  \
            conv_bwd_weight_mfma_kernel<float, TPW, XR, false, false, false, 1, true>                     \
                <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);                                  \
        } else {                                                                                       \
            allow_lds<&conv_bwd_weight_mfma_kernel<bf16, TPW, XR, false, false, false, 1, true>>(b.lds_bytes);   \
            conv_bwd_weight_mfma_kernel<bf16, TPW, XR, false, false, false, 1, true>                      \
                <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);                                  \
        }                                                                                              \
    } while (0)
    int rc = DSK_OK;
    {
        if (b.bf16_cores) {
            rc = launch_bww_bf16(x, dy, (float *)ws, s, st);
            if (rc != DSK_OK) return rc;
        }
        else if (b.fb2) {
            if (in == DSK_F32) {
                allow_lds<&conv_bwd_weight_mfma_kernel<float, 5, 8, false, true, false, 2, true>>(b.lds_bytes);
                conv_bwd_weight_mfma_kernel<float, 5, 8, false, true, false, 2, true>
                    <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);
            } else {
                allow_lds<&conv_bwd_weight_mfma_kernel<bf16, 5, 8, false, true, false, 2, true>>(b.lds_bytes);
                conv_bwd_weight_mfma_kernel<bf16, 5, 8, false, true, false, 2, true>
                    <<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);
            }
        }
        else if (b.packb && b.xrows <= 8) DSK_BW_LAUNCH(2, 8, false, true, true);
        else if (b.packb) DSK_BW_LAUNCH(2, 10, false, true, true);
        else if (b.rowsplit && b.tpw == 1 && b.xrows <= 4) DSK_BW_LAUNCH(1, 4, true, true, false);
        else if (b.rowsplit && b.tpw == 1) DSK_BW_LAUNCH(1, 8, true, true, false);
        else if (b.rowsplit) DSK_BW_LAUNCH(9, 8, true, false, false);
        else if (b.tpw == 1) DSK_BW_LAUNCH(1, 8, false, true, false);
        else if (b.tpw == 2 && b.xrows <= 8) DSK_BW_LAUNCH(2, 8, false, true, false);
        else if (b.tpw == 2) DSK_BW_LAUNCH(2, 10, false, true, false);
        else if (b.tpw == 4) DSK_BW_LAUNCH(4, 8, false, true, false);
        else if (b.tpw == 7 && taps == 25) DSK_BW_LAUNCH_SHARED(7, 8);
        else if (b.tpw == 7) DSK_BW_LAUNCH(7, 8, false, false, false);
        else if (taps == 49) DSK_BW_LAUNCH_SHARED(13, 10);
        else DSK_BW_LAUNCH(13, 10, false, false, false);
        rc = check_launch();
        if (rc != DSK_OK) return rc;
        const long total = (long)s.K * s.C * taps;
        if (b.packb)
            bw_reduce_packb_kernel<<<dim3((unsigned)((total + kRedOut - 1) / kRedOut)), dim3(kThreads), 0, st>>>(
                (const float *)ws, dw, s.K, s.C, s.kh, s.kw, b.Kp, b.n_part);
        else
            bw_reduce_kernel<<<dim3((unsigned)((total + kRedOut - 1) / kRedOut), (unsigned)b.col_passes), dim3(kThreads), 0, st>>>(
                (const float *)ws, dw, s.K, s.C, taps, b.Kp, b.Cp, b.n_part, s.kh * s.kw,
                b.col_passes > 1 ? s.kw : 1, p.pass_stride);
    }
#undef DSK_BW_LAUNCH
#undef DSK_BW_LAUNCH_SHARED
    rc = check_launch();
    if (rc != DSK_OK || !db) return rc;
    float *bpart = (float *)ws + (size_t)b.n_part * b.Kp * b.Cp * (b.packb ? s.kh : taps) * b.col_passes;
    if (in == DSK_F32)
        bias_partial_kernel<float><<<dim3(s.K * kBiasSplit), dim3(kThreads), 0, st>>>((const float *)dy, bpart, s.N,
                                                                                    s.K, (long)s.Ho * s.Wo);
    else
        bias_partial_kernel<bf16><<<dim3(s.K * kBiasSplit), dim3(kThreads), 0, st>>>((const bf16 *)dy, bpart, s.N,
                                                                                   s.K, (long)s.Ho * s.Wo);
    bias_reduce_kernel<<<dim3((s.K + kThreads - 1) / kThreads), dim3(kThreads), 0, st>>>(bpart, db, s.K);
    return check_launch();
}

} // namespace dsk
