// Weight gradient of a stride-1 convolution with a d-regularly sparse kernel (paper Sec. 4.1:
// dw[f][c][a][b] = sum over n, u, v of dy[n][f][u][v] * x[n][c][u+a*d][v+b*d]) for bf16 maps on the
// bf16 matrix cores, square kernels of 1, 3, 4 or 5 taps a side, even tap spacing, maps of even width.
//
// A workgroup owns FB blocks of 32 filters x one block of 32 channels of dw for ALL taps and walks
// over a 1/S share of the pixel tiles (4 rows of one residue class modulo d x 32 columns); its
// partial block goes to the workspace and a second kernel adds the S partial blocks in a fixed
// order.  A = dy (lane = filter), B = x shifted by the tap (lane = channel), and one
// v_mfma_f32_32x32x16_bf16 contracts 16 consecutive pixels of a tile row, of which a lane supplies 8.
// Both tiles lie in LDS as they lie in HBM, [filter or channel][row][column], so they are staged with
// 16-byte loads and 16-byte LDS writes of eight neighbouring pixels (4-byte aligned in HBM, since
// every row starts at an even element) and nothing is transposed.
//
// The accumulator tiles (filter block, tap column b, tap row a) are numbered fblock-major, then b,
// then a, and the four waves take equal contiguous ranges.  Tile row r and tap row a read x-tile row
// r + a, so within a tap column the operand of x row R serves every (r, a) with r + a = R: a wave
// that holds all KH tap rows of a column reads KH + 3 B operands and 4 A operands for 4*KH matrix
// instructions, where one operand pair per instruction would keep LDS busier than the matrix cores.
#include <type_traits>

#include "dsk_internal.h"

namespace dsk {

namespace {

constexpr int kThreads = 256;
constexpr int kXcds = 8;
constexpr int PH = 4, PW = 32;
constexpr int DYB = PH * PW + 8;      // elements per filter of the dy tile: 272 bytes, an odd number of 16-byte units
constexpr int XC = 64;                // columns of the x tile in LDS and as it is staged (eight groups of eight pixels)
constexpr size_t kMaxLds = 64 * 1024;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

struct BbParams {
    const bf16 *x, *dy;
    float *part;         // [split][taps][Kp][Cp]
    int N, C, H, W, K, Ho, Wo, d;
    int Kp, Cp;          // padded to 32
    int xstride;         // elements per channel of the x tile: (PH+k-1) rows of XC columns and 8 more (an odd number of 16-byte
                         // units: 16-byte operand reads), or 4 more (an odd number of 8-byte units: 8- and 4-byte reads)
    int n_rowtile, n_coltile;
    long n_ptile;        // N * n_rowtile * n_coltile
    int S;               // split count
    int n_fgrp, n_cblk;  // groups of FB filter blocks, channel blocks
    int bgroup, bskip;   // image n of x sits at slot n + n / bgroup * bskip (video layers)
    long x_extent;       // readable elements of x
};

// a lane's eight pixels of a B operand; AL: the alignment of the tap columns in pixels
template <int AL>
__device__ inline bf16x8 ld_b(const unsigned short *src)
{
    if constexpr (AL == 8) {
        return *(const bf16x8 *)src;
    } else if constexpr (AL == 4) {
        const u32x2 b0 = *(const u32x2 *)src, b1 = *(const u32x2 *)(src + 4);
        const u32x4 b = {b0[0], b0[1], b1[0], b1[1]};
        return __builtin_bit_cast(bf16x8, b);
    } else {
        const unsigned *s32 = (const unsigned *)src;
        const u32x4 b = {s32[0], s32[1], s32[2], s32[3]};
        return __builtin_bit_cast(bf16x8, b);
    }
}

template <int KH, int KW, int FB, int AL>
__global__ void __launch_bounds__(kThreads, 2)
bww_bf16_kernel(BbParams p)
{
    extern __shared__ __align__(16) unsigned short smem16[];
    unsigned short *dyb = smem16;                      // [32 * FB filters][DYB]
    unsigned short *xb = smem16 + FB * 32 * DYB;       // [32 channels][xstride]
    constexpr int NT = FB * KW * KH;                   // accumulator tiles of the workgroup
    constexpr int MAXT = (NT + 3) / 4;                 // ... of a wave, at most
    constexpr int NDI = 2 * FB;                        // dy items per thread

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lo = lane & 31, hi = lane >> 5;

    // All (filter group, channel block) workgroups of one pixel share are neighbours in the logical
    // order and, through the XCD-aware mapping, run on the same XCD at the same time: the tiles are
    // fetched from HBM once, not once per block.
    const int nblk = p.n_fgrp * p.n_cblk * p.S;
    const int per_xcd = (nblk + kXcds - 1) / kXcds;
    int b = (int)(blockIdx.x % kXcds) * per_xcd + (int)(blockIdx.x / kXcds);
    if (b >= nblk) return;
    const int fg = b % p.n_fgrp; b /= p.n_fgrp;
    const int cb = b % p.n_cblk;
    const int s = b / p.n_cblk;
    const int f_base = fg * 32 * FB;
    const int nf_valid = p.K - f_base, nc_valid = p.C - cb * 32;

    const unsigned HoWo = (unsigned)(p.Ho * p.Wo), dWo = (unsigned)(p.d * p.Wo);
    const unsigned HW = (unsigned)(p.H * p.W), dW = (unsigned)(p.d * p.W);
    const bf16 *dy_end = p.dy + (long)p.N * p.K * HoWo, *x_end = p.x + p.x_extent;

    // dy item i of a thread: filter tid/16 + 16*i, tile row (tid/4)%4, pixel group tid%4
    const int dq_g = tid & 3, dq_r = (tid >> 2) & 3, dq_f = tid >> 4;
    const unsigned dq_off = (unsigned)dq_f * HoWo + (unsigned)dq_r * dWo + 8u * dq_g;
    const int dq_lds = dq_f * DYB + dq_r * PW + 8 * dq_g;
    // x item j of a thread: channel tid/8, tile row j, pixel group tid%8 (a channel beyond C reads the block's first)
    const int xq_c = tid >> 3, xq_g = tid & 7;
    const unsigned xq_off = (xq_c < nc_valid ? (unsigned)xq_c * HW : 0u) + 8u * xq_g;
    const int xq_lds = xq_c * p.xstride + 8 * xq_g;
    constexpr int XR = PH + KH - 1;                    // rows of the x tile

    // Everything from here on is written once per wave number: the accumulator tiles a wave owns, and with them
    // every register index of its matrix loop, differ from wave to wave.  (With only the matrix loop chosen by the
    // wave number inside a common tile loop, the compiler kept the accumulators twice and copied them for every tile.)
    auto run = [&](auto wc) __attribute__((always_inline)) {
    constexpr int W = decltype(wc)::value;
    f32x16 acc[MAXT];
#pragma unroll
    for (int t = 0; t < MAXT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    u32x4 drq[NDI], xrq[XR];
    int st_nr_dy = 0, st_v0 = 0;
    bool st_dy_whole = false;
    // Every tile starts inside both maps (the host enumerates only such tiles), so the tile's base is always a
    // valid address.  Nothing depends on a loaded value before the LDS write, so all loads of a tile are in
    // flight together.  Pixel groups that reach beyond the end of a row read what follows in memory (zero
    // beyond the tensor): dy is masked at the LDS write, x needs no mask (see there).  The x tile is staged
    // XC columns wide whatever the taps need: one item per tile row and thread, with a scalar row offset.
    auto load_tile = [&](long pt) __attribute__((always_inline)) {
        const int ct = (int)(pt % p.n_coltile);
        const int rt = (int)((pt / p.n_coltile) % p.n_rowtile);
        const int n = (int)(pt / ((long)p.n_coltile * p.n_rowtile));
        const int u0 = (rt / p.d) * p.d * PH + (rt % p.d);
        const int v0 = ct * PW;
        const bf16 *dyt = p.dy + (((long)n * p.K + f_base) * p.Ho + u0) * p.Wo + v0;
        const long xn = p.bgroup ? n + (long)(n / p.bgroup) * p.bskip : (long)n;
        const bf16 *xt = p.x + ((xn * p.C + cb * 32) * p.H + u0) * p.W + v0;
        st_nr_dy = (p.Ho - u0 + p.d - 1) / p.d;          // dy rows u0 + r*d that exist (>= 1)
        const int nr_x = (p.H - u0 + p.d - 1) / p.d;     // x rows likewise
        st_v0 = v0;
        st_dy_whole = nf_valid >= 32 * FB && st_nr_dy >= PH;      // every filter and row of the dy tile exists
        const BufRsrc rd = buf_rsrc(dyt, dy_end);
        if (st_dy_whole) {
#pragma unroll
            for (int i = 0; i < NDI; ++i)
                drq[i] = __builtin_amdgcn_raw_buffer_load_b128(rd, (int)(dq_off * 2u), (int)((unsigned)(16 * i) * HoWo * 2u), 0);
        } else {
#pragma unroll
            for (int i = 0; i < NDI; ++i) {
                const bool ok = dq_f + 16 * i < nf_valid && dq_r < st_nr_dy;
                const unsigned off = ok ? dq_off + (unsigned)(16 * i) * HoWo : 0u;
                drq[i] = __builtin_amdgcn_raw_buffer_load_b128(rd, (int)(off * 2u), 0, 0);
            }
        }
        const BufRsrc rx = buf_rsrc(xt, x_end);
#pragma unroll
        for (int j = 0; j < XR; ++j)      // (a row below the map: row 0 is read instead)
            xrq[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(xq_off * 2u), (int)((unsigned)(j < nr_x ? j : 0) * dW * 2u), 0);
    };

    // ---- the matrix instructions of wave W for one staged tile
    auto multiply = [&]() __attribute__((always_inline)) {
        constexpr int T0 = W * NT / 4, T1 = (W + 1) * NT / 4;
        if constexpr (T1 > T0) {      // (fewer tiles than waves, 1 x 1 kernels: a wave without tiles only stages)
        constexpr int CG0 = T0 / KH, CG1 = (T1 - 1) / KH;      // its tap columns (filter block * KW + b)
        constexpr int FK0 = CG0 / KW, FK1 = CG1 / KW;          // its filter blocks
        const unsigned short *al = dyb + lo * DYB + 8 * hi;
        const unsigned short *bl = xb + lo * p.xstride + 8 * hi;
        // tap rows of column cg that belong to this wave
        auto first_a = [](int cg) constexpr { return (T0 > cg * KH ? T0 : cg * KH) - cg * KH; };
        auto last_a = [](int cg) constexpr { return (T1 < (cg + 1) * KH ? T1 : (cg + 1) * KH) - 1 - cg * KH; };
#pragma unroll
        for (int q = 0; q < PW / 16; ++q) {
            bf16x8 A[FK1 - FK0 + 1][PH];
#pragma unroll
            for (int fk = FK0; fk <= FK1; ++fk)
#pragma unroll
                for (int r = 0; r < PH; ++r) A[fk - FK0][r] = *(const bf16x8 *)(al + fk * 32 * DYB + r * PW + 16 * q);
            // The B operand of the next step is read before the matrix instructions of this one are issued, and the
            // scheduler is kept from moving reads across them: moved up, they cost registers the kernel does not have;
            // moved down to their use, their latency is exposed once per step.
            bf16x8 Bc = ld_b<AL>(bl + first_a(CG0) * XC + 16 * q + (CG0 % KW) * p.d), Bn = Bc;
#pragma unroll
            for (int cg = CG0; cg <= CG1; ++cg) {
                const int fk = cg / KW, tb = cg % KW;
                const int a0 = first_a(cg), a1 = last_a(cg);
#pragma unroll
                for (int R = a0; R <= a1 + PH - 1; ++R) {
                    if (R < a1 + PH - 1) Bn = ld_b<AL>(bl + (R + 1) * XC + 16 * q + tb * p.d);
                    else if (cg < CG1) Bn = ld_b<AL>(bl + first_a(cg + 1) * XC + 16 * q + ((cg + 1) % KW) * p.d);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < PH; ++r) {
                        const int a = R - r;
                        if (a >= a0 && a <= a1)
                            acc[cg * KH + a - T0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[fk - FK0][r], Bc, acc[cg * KH + a - T0], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    Bc = Bn;
                }
            }
        }
        }
    };

    long pt = s;
    if (pt < p.n_ptile) load_tile(pt);
    while (pt < p.n_ptile) {
        __syncthreads();        // every wave is done with the previous tile
        {
            const bool cols_whole = st_v0 + PW <= p.Wo;
#pragma unroll
            for (int i = 0; i < NDI; ++i) {
                u32x4 v = drq[i];
                if (!st_dy_whole && !(dq_f + 16 * i < nf_valid && dq_r < st_nr_dy)) v = u32x4{0u, 0u, 0u, 0u};
                if (!cols_whole) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (st_v0 + 8 * dq_g + 2 * k >= p.Wo) v[k] = 0u;      // (the maps are even columns wide)
                }
                *(u32x4 *)(dyb + dq_lds + 16 * i * DYB) = v;
            }
            // No zeroing of x: an x entry outside the map (some finite value of the tensor was read instead) only ever
            // meets dy entries outside THEIR map, which are zeros, and the columns of channels beyond C are never
            // written out.
#pragma unroll
            for (int j = 0; j < XR; ++j) {
                if constexpr (AL == 8) {
                    *(u32x4 *)(xb + xq_lds + j * XC) = xrq[j];
                } else {      // (the channels are 8-byte aligned only)
                    *(u32x2 *)(xb + xq_lds + j * XC) = u32x2{xrq[j][0], xrq[j][1]};
                    *(u32x2 *)(xb + xq_lds + j * XC + 4) = u32x2{xrq[j][2], xrq[j][3]};
                }
            }
        }
        __syncthreads();
        if (pt + p.S < p.n_ptile) load_tile(pt + p.S);      // in flight while the matrix cores run
        pt += p.S;
        multiply();
    }

    // ---- partial block out: part[split][tap][f][c]; lane = channel, registers = filters
    float *part = p.part + (long)s * p.Kp * p.Cp * (KH * KW);
    {
        constexpr int T0 = W * NT / 4, T1 = (W + 1) * NT / 4;
#pragma unroll
        for (int t = T0; t < T1; ++t) {
            const int cg = t / KH, a = t % KH, fk = cg / KW, tb = cg % KW;
            if (f_base + fk * 32 >= p.Kp) continue;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int f = f_base + fk * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
                part[((long)(a * KW + tb) * p.Kp + f) * p.Cp + cb * 32 + lo] = acc[t - T0][i];      // 32 consecutive channels per store
            }
        }
    }
    };
    switch (wave) {
    case 0: run(std::integral_constant<int, 0>{}); break;
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: run(std::integral_constant<int, 2>{}); break;
    default: run(std::integral_constant<int, 3>{}); break;
    }
}

struct BbPlan {
    bool ok;
    int k, d, FB, AL, Kp, Cp, xstride, n_rowtile, n_coltile, S, n_fgrp, n_cblk;
    long n_ptile;
    size_t lds_bytes;
};

BbPlan bb_plan(const ConvShape &s)
{
    BbPlan b{};
    if (s.kh != s.kw || !(s.kh == 1 || (s.kh >= 3 && s.kh <= 5))) return b;
    if ((s.d % 2 != 0 && s.kh > 1) || s.W % 2 != 0 || s.gsize != 0) return b;
    if ((long)s.H * s.W >= (1L << 24)) return b;      // 32-channel block offsets stay below 2^29 elements
    b.k = s.kh;
    b.d = s.kh == 1 ? 1 : s.d;      // a 1 x 1 kernel has no taps to space: tiles of neighbouring rows
    b.Kp = (s.K + 31) / 32 * 32;
    b.Cp = (s.C + 31) / 32 * 32;
    const int n_fblk = b.Kp / 32;
    b.n_cblk = b.Cp / 32;
    if (PW + (s.kw - 1) * s.d > XC) return b;         // the taps reach beyond the x tile
    b.AL = s.kh == 1 || s.d % 8 == 0 ? 8 : s.d % 4 == 0 ? 4 : 2;
    // narrower operand reads: channels an odd number of 8-byte units apart spread the lanes over twice as many banks
    b.xstride = (PH + s.kh - 1) * XC + (b.AL == 8 ? 8 : 4);
    // filter blocks per workgroup: as many as give every wave whole tap columns
    b.FB = s.kh == 5 ? 1 : s.kh == 4 ? (n_fblk >= 2 ? 2 : 1) : (n_fblk >= 3 ? 4 : n_fblk == 2 ? 2 : 1);      // (1 x 1: a block per wave)
    for (;; b.FB /= 2) {
        b.lds_bytes = 2 * ((size_t)b.FB * 32 * DYB + (size_t)32 * b.xstride);
        // (a thread's dy offsets span 32*FB planes and are taken as 32-bit byte offsets)
        if (b.lds_bytes <= kMaxLds && (long)32 * b.FB * s.Ho * s.Wo * 2 < (1L << 31)) break;
        if (b.FB == 1) return b;
    }
    b.n_fgrp = (n_fblk + b.FB - 1) / b.FB;
    // residue classes of the last row block that start beyond the map hold no pixel: skip them
    {
        const int nrb = (s.Ho + b.d * PH - 1) / (b.d * PH);
        const int last = s.Ho - (nrb - 1) * b.d * PH;
        b.n_rowtile = (nrb - 1) * b.d + (last < b.d ? last : b.d);
    }
    b.n_coltile = (s.Wo + PW - 1) / PW;
    b.n_ptile = (long)s.N * b.n_rowtile * b.n_coltile;
    const long blocks = (long)b.n_fgrp * b.n_cblk;
    long S = 2048 / blocks;
    if (S > 256) S = 256;
    if (S > b.n_ptile / 4) S = b.n_ptile / 4;
    if (S < 1) S = 1;
    b.S = (int)S;
    b.ok = true;
    return b;
}

template <int K, int FB>
void bb_launch_al(const BbParams &p, int al, unsigned grid, size_t lds, hipStream_t st)
{
    if (al == 8) bww_bf16_kernel<K, K, FB, 8><<<dim3(grid), dim3(kThreads), lds, st>>>(p);
    else if (al == 4) bww_bf16_kernel<K, K, FB, 4><<<dim3(grid), dim3(kThreads), lds, st>>>(p);
    else bww_bf16_kernel<K, K, FB, 2><<<dim3(grid), dim3(kThreads), lds, st>>>(p);
}

} // namespace

bool bww_bf16_shape(const ConvShape &s, int *Kp, int *Cp, int *S)
{
    const BbPlan b = bb_plan(s);
    if (!b.ok) return false;
    *Kp = b.Kp; *Cp = b.Cp; *S = b.S;
    return true;
}

int launch_bww_bf16(const void *x, const void *dy, float *part, const ConvShape &s, hipStream_t st)
{
    const BbPlan b = bb_plan(s);
    if (!b.ok) return DSK_ESHAPE;
    BbParams p{};
    p.x = (const bf16 *)x; p.dy = (const bf16 *)dy; p.part = part;
    p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.Ho = s.Ho; p.Wo = s.Wo; p.d = b.d;
    p.Kp = b.Kp; p.Cp = b.Cp; p.xstride = b.xstride;
    p.n_rowtile = b.n_rowtile; p.n_coltile = b.n_coltile; p.n_ptile = b.n_ptile; p.S = b.S;
    p.n_fgrp = b.n_fgrp; p.n_cblk = b.n_cblk;
    p.bgroup = s.bgroup; p.bskip = s.bskip;
    p.x_extent = s.in_extent ? s.in_extent : (long)s.N * s.C * s.H * s.W;
    const unsigned grid = (unsigned)(((long)b.n_fgrp * b.n_cblk * b.S + kXcds - 1) / kXcds * kXcds);
    if (b.k == 3 && b.FB == 4) bb_launch_al<3, 4>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.k == 3 && b.FB == 2) bb_launch_al<3, 2>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.k == 3) bb_launch_al<3, 1>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.k == 4 && b.FB == 2) bb_launch_al<4, 2>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.k == 4) bb_launch_al<4, 1>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.k == 5) bb_launch_al<5, 1>(p, b.AL, grid, b.lds_bytes, st);
    else if (b.FB == 4) bww_bf16_kernel<1, 1, 4, 8><<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);
    else if (b.FB == 2) bww_bf16_kernel<1, 1, 2, 8><<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);
    else bww_bf16_kernel<1, 1, 1, 8><<<dim3(grid), dim3(kThreads), b.lds_bytes, st>>>(p);
    return check_launch();
}

} // namespace dsk
