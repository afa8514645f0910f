// Stride-1 pooling with d-regularly sparse k x k kernels (paper Sec. 3.1-3.2;
// backward Sec. 4.2).  Bandwidth-bound: every input element should come from
// HBM once.  A thread owns V neighbouring columns and R output rows that lie in
// ONE residue class modulo d (rows u0, u0+d, u0+2d, ...): the k taps of
// neighbouring outputs in that class share input rows, so R outputs need R+k-1
// row visits instead of R*k, and every wavefront load is one contiguous row
// segment.  Column taps (v, v+d, ...) of a wavefront overlap in the same cache
// lines.
//
// V = 2 (maps of even width, even d): a lane moves two pixels per memory
// instruction.  The vector memory path takes about 16 cycles per wavefront
// instruction whatever its width up to 16 bytes per lane, which bounds kernels
// that move few bytes per instruction: bf16 maps, and the max-pool gradient
// with its one-byte tap indices.
//
// Max-pool ties: taps are ranked by a*k+b and only a strictly greater value
// replaces the running maximum, so the lowest index wins.  Taking the first
// maximum of each input row and then the first row holding the overall maximum
// selects exactly that tap.
#include "dsk_internal.h"
#include <utility>

namespace dsk {

static constexpr int kPoolThreads = 256;
static constexpr int kPoolXcds = 8;
typedef unsigned pool_u32x2 __attribute__((ext_vector_type(2)));
typedef float pool_f32x2 __attribute__((ext_vector_type(2)));

struct PoolShape {
    int planes, H, W, Ho, Wo, k, d;
    int col_blocks, row_groups;   // row_groups = ceil(rows / (d*R)) * d
    int cl_log2;                  // 64, 128 or 256 threads of a workgroup lie side by side along a row ...
    int row_blocks;               // ... and the 4, 2 or 1 such runs take consecutive row groups
    long n_blocks;                // planes * row_blocks * col_blocks
    long per_xcd;                 // the grid is 8 * per_xcd workgroups
    int rr;                       // 1: workgroup i takes tile i; 0: every XCD takes one contiguous run of tiles
};

// Decode blockIdx.x -> (plane, first row of the residue class, first column); false: no such row group.
template <int R, int V>
__device__ inline bool pool_decode(const PoolShape &s, int &plane, int &r0, int &col)
{
    // Consecutive workgroups of a grid go to different XCDs, each with an L2 of its own; rr = 0
    // gives every XCD one contiguous run of tiles instead.
    long b = s.rr ? (long)blockIdx.x : (long)(blockIdx.x % kPoolXcds) * s.per_xcd + blockIdx.x / kPoolXcds;
    if (b >= s.n_blocks) return false;
    const int cb = (int)(b % s.col_blocks);
    b /= s.col_blocks;
    const int rb = (int)(b % s.row_blocks);
    plane = (int)(b / s.row_blocks);
    // (a run is at least one wave long: the row group is uniform over a wave, and the compiler has to know)
    const int rg = rb * (kPoolThreads >> s.cl_log2) + __builtin_amdgcn_readfirstlane((int)threadIdx.x >> s.cl_log2);
    const int grp = rg / s.d, res = rg % s.d;
    r0 = grp * s.d * R + res;
    col = ((cb << s.cl_log2) + ((int)threadIdx.x & ((1 << s.cl_log2) - 1))) * V;
    return rg < s.row_groups;
}

// V neighbouring elements with one buffer access (element offsets; for V = 2 the sum of the
// offsets is even, so the access is naturally aligned)
template <int V>
__device__ inline void pool_ld(BufRsrc r, const float *p, unsigned lane_off, unsigned uniform_off, float (&o)[V])
{
    if constexpr (V == 1) {
        o[0] = buf_ld(r, p, lane_off, uniform_off);
    } else {
        // (the whole vector is converted: __builtin_bit_cast of a vector ELEMENT reads element 0 whichever is named)
        const pool_f32x2 t = __builtin_bit_cast(pool_f32x2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)(lane_off * 4u), (int)(uniform_off * 4u), 0));
        o[0] = t[0];
        o[1] = t[1];
    }
}
template <int V>
__device__ inline void pool_ld(BufRsrc r, const bf16 *p, unsigned lane_off, unsigned uniform_off, float (&o)[V])
{
    if constexpr (V == 1) {
        o[0] = buf_ld(r, p, lane_off, uniform_off);
    } else {
        const unsigned t = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r, (int)(lane_off * 2u), (int)(uniform_off * 2u), 0);
        o[0] = __builtin_bit_cast(float, t << 16);
        o[1] = __builtin_bit_cast(float, t & 0xffff0000u);
    }
}
// V tap indices, one per byte of the result
template <int V>
__device__ inline int pool_ld_idx(BufRsrc r, const uint8_t *p, unsigned lane_off, unsigned uniform_off)
{
    if constexpr (V == 1) return buf_ld(r, p, lane_off, uniform_off);
    else return (int)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)lane_off, (int)uniform_off, 0);
}
template <int V>
__device__ inline void pool_st(BufRsrc r, float *p, unsigned lane_off, unsigned uniform_off, const float (&v)[V])
{
    if constexpr (V == 1) {
        buf_st(r, p, lane_off, uniform_off, v[0]);
    } else {
        const pool_f32x2 t = {v[0], v[1]};
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(pool_u32x2, t), r, (int)(lane_off * 4u), (int)(uniform_off * 4u), 0);
    }
}
template <int V>
__device__ inline void pool_st(BufRsrc r, bf16 *p, unsigned lane_off, unsigned uniform_off, const float (&v)[V])
{
    if constexpr (V == 1) {
        buf_st(r, p, lane_off, uniform_off, v[0]);
    } else {
        const unsigned t = (unsigned)f32_to_bf16(v[0]).v | (unsigned)f32_to_bf16(v[1]).v << 16;
        __builtin_amdgcn_raw_buffer_store_b32(t, r, (int)(lane_off * 2u), (int)(uniform_off * 2u), 0);
    }
}
template <int V>
__device__ inline void pool_st_idx(BufRsrc r, uint8_t *p, unsigned lane_off, unsigned uniform_off, const int (&v)[V])
{
    if constexpr (V == 1) buf_st(r, p, lane_off, uniform_off, v[0]);
    else __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(v[0] | v[1] << 8), r, (int)lane_off, (int)uniform_off, 0);
}

// All loads of a thread are issued before anything depends on one of them: rows and columns
// that do not exist are clamped to ones that do (their values are never used), so no load sits
// under a condition, and every access is a buffer access with one per-lane offset per tap
// column and a scalar offset per row.
template <typename T, int K, int R, bool IS_MAX, int V>
__global__ void __launch_bounds__(kPoolThreads)
pool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    int plane, u0, v;
    if (!pool_decode<R, V>(s, plane, u0, v) || u0 >= s.Ho) return;
    const bool col_ok = v < s.Wo;                 // V = 2: Wo is even, both columns exist or neither
    unsigned vc = col_ok ? (unsigned)v : 0u;      // column 0 exists; v + b*d < W whenever v < Wo
    const T *xp = x + (long)plane * s.H * s.W;
    const BufRsrc rx = buf_rsrc(xp, xp + (long)s.H * s.W);
    // rows per batch of loads: all of them for small windows; one row (K loads) for large ones,
    // which would otherwise need (R+K-1)*K registers
    constexpr int NT = R + K - 1, TB = K <= 3 ? NT : 1;
    float rowv[NT][V];
    int rowi[NT][V];
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += TB) {
        float xv[TB][K][V];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            int row = u0 + (t0 + t) * s.d;
            row = row < s.H ? row : s.H - 1;
#pragma unroll
            for (int b = 0; b < K; ++b) pool_ld<V>(rx, xp, vc + (unsigned)(b * s.d), (unsigned)(row * s.W), xv[t][b]);
        }
        // the values are pinned here so that the loads of a batch are issued together above,
        // not one by one where the branches below use them
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int b = 0; b < K; ++b)
#pragma unroll
                for (int j = 0; j < V; ++j) asm volatile("" : "+v"(xv[t][b][j]));
        // ... and the next batch is not hoisted above this one (its offset "changes" here)
        if (TB < NT) asm volatile("" : "+v"(vc));
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float best = xv[t][0][j];
                int bi = 0;
#pragma unroll
                for (int b = 1; b < K; ++b) {
                    if (IS_MAX) {
                        if (xv[t][b][j] > best) { best = xv[t][b][j]; bi = b; }
                    } else {
                        best += xv[t][b][j];
                    }
                }
                rowv[t0 + t][j] = best;
                rowi[t0 + t][j] = bi;
            }
    }
    if (!col_ok) return;
    T *yp = y + (long)plane * s.Ho * s.Wo;
    const BufRsrc ry = buf_rsrc(yp, yp + (long)s.Ho * s.Wo);
    uint8_t *ap = IS_MAX && am ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc ra = buf_rsrc(ap, ap + (ap ? (long)s.Ho * s.Wo : 0));
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int u = u0 + r * s.d;
        if (u >= s.Ho) break;
        float best[V];
        int bi[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            best[j] = rowv[r][j];
            bi[j] = rowi[r][j];
            if (IS_MAX) {
#pragma unroll
                for (int a = 1; a < K; ++a)
                    if (rowv[r + a][j] > best[j]) { best[j] = rowv[r + a][j]; bi[j] = a * K + rowi[r + a][j]; }
            } else {
#pragma unroll
                for (int a = 1; a < K; ++a) best[j] += rowv[r + a][j];
                best[j] *= 1.0f / (float)(K * K);
            }
        }
        pool_st<V>(ry, yp, (unsigned)v, (unsigned)(u * s.Wo), best);
        if (ap) pool_st_idx<V>(ra, ap, (unsigned)v, (unsigned)(u * s.Wo), bi);
    }
}

// dx rows p0 + r*d (r < R) of V columns: they collect from dy rows p0 + (r-a)*d.
template <typename T, int K, int R, bool IS_MAX, int V>
__global__ void __launch_bounds__(kPoolThreads)
pool_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, PoolShape s)
{
    int plane, p0, q;
    if (!pool_decode<R, V>(s, plane, p0, q) || p0 >= s.H) return;
    const bool col_ok = q < s.W;                  // V = 2: W is even, both columns exist or neither
    const T *dyp = dy + (long)plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc rg = buf_rsrc(dyp, dyp + (long)s.Ho * s.Wo);
    const BufRsrc ra = buf_rsrc(amp, amp + (IS_MAX ? (long)s.Ho * s.Wo : 0));
    // dy column q - b*d, clamped into the map; `cok` bit b says that it exists (V = 2: q, d and Wo
    // are even, so columns q - b*d and q - b*d + 1 exist together)
    unsigned vcol[K];
    unsigned cok = 0;
#pragma unroll
    for (int b = 0; b < K; ++b) {
        const int v = q - b * s.d;
        const bool ok = col_ok && v >= 0 && v < s.Wo;
        vcol[b] = ok ? (unsigned)v : 0u;
        cok |= ok ? 1u << b : 0u;
    }
    // t indexes dy rows p0 + (t-(K-1))*d, t = 0 .. R+K-2; it feeds dx rows r = t-(K-1)+a.
    // Rows per batch of loads: all of them for small windows, one row (2K loads) for large ones.
    constexpr int NT = R + K - 1, TB = K <= 3 ? NT : 1;
    float acc[R][V];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < V; ++j) acc[r][j] = 0.f;
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += TB) {
        float g[TB][K][V];
        int idx[TB][K];       // one tap index per byte
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            int u = p0 + (t0 + t - (K - 1)) * s.d;
            u = u < 0 ? 0 : (u >= s.Ho ? s.Ho - 1 : u);
#pragma unroll
            for (int b = 0; b < K; ++b) {
                pool_ld<V>(rg, dyp, vcol[b], (unsigned)(u * s.Wo), g[t][b]);
                idx[t][b] = IS_MAX ? pool_ld_idx<V>(ra, amp, vcol[b], (unsigned)(u * s.Wo)) : 0;
            }
        }
        // the values are pinned here so that the loads of a batch are issued together above,
        // not one by one where the branches below use them
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int b = 0; b < K; ++b) {
#pragma unroll
                for (int j = 0; j < V; ++j) asm volatile("" : "+v"(g[t][b][j]));
                if (IS_MAX) asm volatile("" : "+v"(idx[t][b]));
            }
        // ... and the next batch is not hoisted above this one (its offsets "change" here):
        // one batch in flight per wave keeps the register count, and with it the occupancy, sane
        if (TB < NT)
#pragma unroll
            for (int b = 0; b < K; ++b) asm volatile("" : "+v"(vcol[b]));
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const int u = p0 + (t0 + t - (K - 1)) * s.d;
            const bool row_ok = u >= 0 && u < s.Ho;       // uniform
#pragma unroll
            for (int b = 0; b < K; ++b)
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    const float gv = row_ok && ((cok >> b) & 1u) ? g[t][b][j] : 0.f;
                    const int tap = (idx[t][b] >> (8 * j)) & 0xff;
#pragma unroll
                    for (int a = 0; a < K; ++a) {
                        const int r = t0 + t - (K - 1) + a;
                        if (r >= 0 && r < R) acc[r][j] += !IS_MAX || tap == a * K + b ? gv : 0.f;
                    }
                }
        }
    }
    if (!col_ok) return;
    T *dxp = dx + (long)plane * s.H * s.W;
    const BufRsrc rd = buf_rsrc(dxp, dxp + (long)s.H * s.W);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = p0 + r * s.d;
        if (p >= s.H) break;
        float v[V];
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = IS_MAX ? acc[r][j] : acc[r][j] * (1.0f / (float)(K * K));
        pool_st<V>(rd, dxp, (unsigned)q, (unsigned)(p * s.W), v);
    }
}

// ---- d = 1, k = 4 or 8, fp32: the taps of a row are neighbours in memory ----
// A thread owns FOUR neighbouring columns and R consecutive rows.  For one input row it needs the
// k + 3 pixels from its first column on: two or three 16-byte loads instead of 4k scalar ones.
// The kernels above spend (R+k-1)*k load instructions on R outputs, and with k = 8 that, at about
// 16 cycles of the vector memory path per wavefront instruction, is what bounds them.
typedef float pool_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned pool_u32x4 __attribute__((ext_vector_type(4)));

template <int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_span_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    constexpr int V = 4, NS = (V + K - 1 + 3) / 4, NT = R + K - 1;
    int plane, u0, v;
    if (!pool_decode<R, V>(s, plane, u0, v) || u0 >= s.Ho || v >= s.Wo) return;
    const float *xp = x + (long)plane * s.H * s.W;
    const BufRsrc rx = buf_rsrc(xp, xp + (long)s.H * s.W);
    unsigned vc = (unsigned)v;            // v < Wo: the first pixel exists; what a load reads beyond the row's end
                                          // (the next row, or zero beyond the plane) only reaches columns >= Wo
    float rowv[NT][V];
    int rowi[NT][V];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int row = u0 + t;
        row = row < s.H ? row : s.H - 1;
        pool_f32x4 sp[NS];
#pragma unroll
        for (int i = 0; i < NS; ++i)
            sp[i] = __builtin_bit_cast(pool_f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)((vc + 4u * i) * 4u), (int)((unsigned)(row * s.W) * 4u), 0));
#pragma unroll
        for (int i = 0; i < NS; ++i) asm volatile("" : "+v"(sp[i]));
        asm volatile("" : "+v"(vc));      // one row's loads in flight per wave at a time
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float best = sp[j / 4][j % 4];
            int bi = 0;
#pragma unroll
            for (int b = 1; b < K; ++b) {
                const float c = sp[(j + b) / 4][(j + b) % 4];
                if (IS_MAX) {
                    if (c > best) { best = c; bi = b; }
                } else {
                    best += c;
                }
            }
            rowv[t][j] = best;
            rowi[t][j] = bi;
        }
    }
    float *yp = y + (long)plane * s.Ho * s.Wo;
    const BufRsrc ry = buf_rsrc(yp, yp + (long)s.Ho * s.Wo);
    uint8_t *ap = IS_MAX && am ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc ra = buf_rsrc(ap, ap + (ap ? (long)s.Ho * s.Wo : 0));
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int u = u0 + r;
        if (u >= s.Ho) break;
        float best[V];
        int bi[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            best[j] = rowv[r][j];
            bi[j] = rowi[r][j];
            if (IS_MAX) {
#pragma unroll
                for (int a = 1; a < K; ++a)
                    if (rowv[r + a][j] > best[j]) { best[j] = rowv[r + a][j]; bi[j] = a * K + rowi[r + a][j]; }
            } else {
#pragma unroll
                for (int a = 1; a < K; ++a) best[j] += rowv[r + a][j];
                best[j] *= 1.0f / (float)(K * K);
            }
        }
        const unsigned ro = (unsigned)(u * s.Wo);
        if (v + V <= s.Wo) {
            const pool_f32x4 o = {best[0], best[1], best[2], best[3]};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(pool_u32x4, o), ry, (int)((unsigned)v * 4u), (int)(ro * 4u), 0);
            if (ap) {
                if ((ro & 3u) == 0) {      // uniform: the four tap indices are one aligned word
                    const unsigned w = (unsigned)bi[0] | (unsigned)bi[1] << 8 | (unsigned)bi[2] << 16 | (unsigned)bi[3] << 24;
                    __builtin_amdgcn_raw_buffer_store_b32(w, ra, v, (int)ro, 0);
                } else {
#pragma unroll
                    for (int j = 0; j < V; ++j) buf_st(ra, ap, (unsigned)(v + j), ro, bi[j]);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (v + j < s.Wo) {
                    buf_st(ry, yp, (unsigned)(v + j), ro, best[j]);
                    if (ap) buf_st(ra, ap, (unsigned)(v + j), ro, bi[j]);
                }
        }
    }
}

// The gradient (Wo a multiple of 4, so that the four tap indices of an aligned group of dy columns
// are one aligned word): dx columns q .. q+3 collect from dy columns q-(K-1) .. q+3, read as the
// aligned groups from column q - KP on, KP = K-1 rounded up to 4.
//
// One dy row: row p0 + T - (K-1) feeds dx row p0 + r through tap row a = r - T + K-1, and dx column
// q + j takes dy column q + j - b through tap column b.  T is a template argument (the rows are
// enumerated by a fold expression): the k*k*R tests per thread are too many for the loop unroller.
template <int K, int R, bool IS_MAX, int T>
__device__ __attribute__((always_inline)) inline void pool_span_bwd_row(const PoolShape &s, BufRsrc rg, BufRsrc ra, int p0,
                                                                        unsigned (&voff)[(K - 1 + 3) / 4 + 1], unsigned gok,
                                                                        float (&acc)[R][4])
{
    constexpr int V = 4, KP = (K - 1 + 3) / 4 * 4, NS = KP / 4 + 1;
    const int u = p0 + T - (K - 1);
    const bool row_ok = u >= 0 && u < s.Ho;       // uniform
    const unsigned ro = (unsigned)((u < 0 ? 0 : (u >= s.Ho ? s.Ho - 1 : u)) * s.Wo);
    pool_f32x4 g[NS];
    unsigned id[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        g[i] = __builtin_bit_cast(pool_f32x4, __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(voff[i] * 4u), (int)(ro * 4u), 0));
        id[i] = IS_MAX ? (unsigned)__builtin_amdgcn_raw_buffer_load_b32(ra, (int)voff[i], (int)ro, 0) : 0u;
    }
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        asm volatile("" : "+v"(g[i]));
        if (IS_MAX) asm volatile("" : "+v"(id[i]));
    }
#pragma unroll
    for (int i = 0; i < NS; ++i) asm volatile("" : "+v"(voff[i]));      // one row's loads in flight per wave
    float gm[4 * NS];     // element n = dy column q - KP + n, zero where it does not exist
    int tap[4 * NS];
#pragma unroll
    for (int n = 0; n < 4 * NS; ++n) {
        gm[n] = row_ok && ((gok >> (n / 4)) & 1u) ? g[n / 4][n % 4] : 0.f;
        tap[n] = (int)((id[n / 4] >> (8 * (n % 4))) & 0xffu);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        constexpr int a0 = K - 1 - T;
        const int a = r + a0;
        if (a < 0 || a >= K) continue;
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int b = 0; b < K; ++b) acc[r][j] += !IS_MAX || tap[KP + j - b] == a * K + b ? gm[KP + j - b] : 0.f;
    }
    // a row is finished before the next one starts: interleaved, the rows need every register of the SIMD
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < V; ++j) asm volatile("" : "+v"(acc[r][j]));
}

template <int K, int R, bool IS_MAX, int... Ts>
__device__ __attribute__((always_inline)) inline void pool_span_bwd_rows(const PoolShape &s, BufRsrc rg, BufRsrc ra, int p0,
                                                                         unsigned (&voff)[(K - 1 + 3) / 4 + 1], unsigned gok,
                                                                         float (&acc)[R][4], std::integer_sequence<int, Ts...>)
{
    (pool_span_bwd_row<K, R, IS_MAX, Ts>(s, rg, ra, p0, voff, gok, acc), ...);
}

template <int K, int R, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_span_bwd_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ am, float *__restrict__ dx, PoolShape s)
{
    constexpr int V = 4, KP = (K - 1 + 3) / 4 * 4, NS = KP / 4 + 1, NT = R + K - 1;
    int plane, p0, q;
    if (!pool_decode<R, V>(s, plane, p0, q) || p0 >= s.H || q >= s.W) return;
    const float *dyp = dy + (long)plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + (long)plane * s.Ho * s.Wo : nullptr;
    const BufRsrc rg = buf_rsrc(dyp, dyp + (long)s.Ho * s.Wo);
    const BufRsrc ra = buf_rsrc(amp, amp + (IS_MAX ? (long)s.Ho * s.Wo : 0));
    // group i = dy columns q - KP + 4i .. + 3: all four exist or none (q and Wo are multiples of 4)
    unsigned voff[NS];
    unsigned gok = 0;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int c = q - KP + 4 * i;
        const bool ok = c >= 0 && c < s.Wo;
        voff[i] = ok ? (unsigned)c : 0u;
        gok |= ok ? 1u << i : 0u;
    }
    float acc[R][V];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < V; ++j) acc[r][j] = 0.f;
    pool_span_bwd_rows<K, R, IS_MAX>(s, rg, ra, p0, voff, gok, acc, std::make_integer_sequence<int, NT>{});
    float *dxp = dx + (long)plane * s.H * s.W;
    const BufRsrc rd = buf_rsrc(dxp, dxp + (long)s.H * s.W);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = p0 + r;
        if (p >= s.H) break;
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = IS_MAX ? acc[r][j] : acc[r][j] * (1.0f / (float)(K * K));
        const unsigned ro = (unsigned)(p * s.W);
        if (q + V <= s.W) {
            const pool_f32x4 w = {o[0], o[1], o[2], o[3]};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(pool_u32x4, w), rd, (int)((unsigned)q * 4u), (int)(ro * 4u), 0);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (q + j < s.W) buf_st(rd, dxp, (unsigned)(q + j), ro, o[j]);
        }
    }
}

// ---- any k: one thread per output entry ----
template <typename T, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_fwd_generic_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ am, PoolShape s)
{
    const long total = (long)s.planes * s.Ho * s.Wo;
    const long idx = (long)blockIdx.x * kPoolThreads + threadIdx.x;
    if (idx >= total) return;
    const int v = (int)(idx % s.Wo);
    const int u = (int)((idx / s.Wo) % s.Ho);
    const long plane = idx / ((long)s.Wo * s.Ho);
    const T *xp = x + (plane * s.H + u) * s.W + v;
    float best = ldf(xp, 0);
    int bi = 0;
    for (int a = 0; a < s.k; ++a)
        for (int b = 0; b < s.k; ++b) {
            if (a == 0 && b == 0) continue;
            const float t = ldf(xp, (long)a * s.d * s.W + b * s.d);
            if (IS_MAX) {
                if (t > best) { best = t; bi = a * s.k + b; }
            } else {
                best += t;
            }
        }
    if (!IS_MAX) best *= 1.0f / (float)(s.k * s.k);
    stf(y, idx, best);
    if (IS_MAX && am) am[idx] = (uint8_t)bi;
}

template <typename T, bool IS_MAX>
__global__ void __launch_bounds__(kPoolThreads)
pool_bwd_generic_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ am, T *__restrict__ dx, PoolShape s)
{
    const long total = (long)s.planes * s.H * s.W;
    const long idx = (long)blockIdx.x * kPoolThreads + threadIdx.x;
    if (idx >= total) return;
    const int q = (int)(idx % s.W);
    const int p = (int)((idx / s.W) % s.H);
    const long plane = idx / ((long)s.W * s.H);
    const T *dyp = dy + plane * s.Ho * s.Wo;
    const uint8_t *amp = IS_MAX ? am + plane * s.Ho * s.Wo : nullptr;
    float acc = 0.f;
    for (int a = 0; a < s.k; ++a) {
        const int u = p - a * s.d;
        if (u < 0 || u >= s.Ho) continue;
        for (int b = 0; b < s.k; ++b) {
            const int v = q - b * s.d;
            if (v < 0 || v >= s.Wo) continue;
            const long o = (long)u * s.Wo + v;
            if (IS_MAX) {
                if (amp[o] == a * s.k + b) acc += ldf(dyp, o);
            } else {
                acc += ldf(dyp, o);
            }
        }
    }
    if (!IS_MAX) acc *= 1.0f / (float)(s.k * s.k);
    stf(dx, idx, acc);
}

// rows / cols: extent of the map the threads are spread over; V columns per thread
static PoolShape make_shape(int N, int C, int H, int W, int k, int d, int R, int rows, int cols, int V)
{
    PoolShape s;
    s.planes = N * C;
    s.H = H; s.W = W;
    s.Ho = H - (k - 1) * d; s.Wo = W - (k - 1) * d;
    s.k = k; s.d = d;
    // Threads side by side along a row, and the placement of the workgroups.  Measured inside a
    // network step (the map has just been written by a convolution): with one pixel per thread,
    // 1 KB of a row per workgroup and round-robin placement are fastest; with pixel pairs, the
    // run length that leaves the fewest threads beyond the map and one contiguous run of tiles
    // per XCD, whose L2 then serves the rows and columns neighbouring tiles share.
    const int lanes = (cols + V - 1) / V;
    s.cl_log2 = 8;
    s.rr = V == 1;
    for (int l = 7; l >= 6 && V > 1; --l)
        if (((lanes + (1 << l) - 1) >> l << l) < ((lanes + (1 << s.cl_log2) - 1) >> s.cl_log2 << s.cl_log2)) s.cl_log2 = l;
    s.col_blocks = (lanes + (1 << s.cl_log2) - 1) >> s.cl_log2;
    s.row_groups = ((rows + d * R - 1) / (d * R)) * d;
    const int runs = kPoolThreads >> s.cl_log2;
    s.row_blocks = (s.row_groups + runs - 1) / runs;
    s.n_blocks = (long)s.planes * s.row_blocks * s.col_blocks;
    s.per_xcd = (s.n_blocks + kPoolXcds - 1) / kPoolXcds;
    return s;
}

template <typename T, bool IS_MAX, int V>
static int pool_fwd_dispatch(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                             hipStream_t st)
{
    constexpr int R = 8;
    PoolShape s = make_shape(N, C, H, W, k, d, R, H - (k - 1) * d, W - (k - 1) * d, V);
    const long tiled_blocks = s.per_xcd * kPoolXcds;
    if (k == 2 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 2, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 3 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 3, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 4 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 4, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else if (k == 8 && tiled_blocks < 0x7fffffffL)
        pool_fwd_kernel<T, 8, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)x, (T *)y, am, s);
    else {
        const long total = (long)s.planes * s.Ho * s.Wo;
        pool_fwd_generic_kernel<T, IS_MAX>
            <<<dim3((unsigned)((total + kPoolThreads - 1) / kPoolThreads)), dim3(kPoolThreads), 0, st>>>(
                (const T *)x, (T *)y, am, s);
    }
    return check_launch();
}

template <typename T, bool IS_MAX, int V>
static int pool_bwd_dispatch(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k,
                             int d, hipStream_t st)
{
    // rows per thread: 8 for small windows; 2 for 4x4 and 8x8 ones, whose k*k tests per row pair
    // otherwise unroll into a kernel that needs every register of the SIMD
    constexpr int R = 8, RL = 2;
    PoolShape s = make_shape(N, C, H, W, k, d, k <= 3 ? R : RL, H, W, V);
    const long tiled_blocks = s.per_xcd * kPoolXcds;
    if (k == 2 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 2, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 3 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 3, R, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 4 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 4, RL, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else if (k == 8 && tiled_blocks < 0x7fffffffL)
        pool_bwd_kernel<T, 8, RL, IS_MAX, V><<<dim3((unsigned)tiled_blocks), dim3(kPoolThreads), 0, st>>>(
            (const T *)dy, am, (T *)dx, s);
    else {
        const long total = (long)s.planes * s.H * s.W;
        pool_bwd_generic_kernel<T, IS_MAX>
            <<<dim3((unsigned)((total + kPoolThreads - 1) / kPoolThreads)), dim3(kPoolThreads), 0, st>>>(
                (const T *)dy, am, (T *)dx, s);
    }
    return check_launch();
}

// two pixels per thread and memory instruction need pixel pairs that are aligned in every row and at every tap
static bool pool_pairs(int W, int d) { return W % 2 == 0 && d % 2 == 0; }

static constexpr int kSpanR = 4;      // rows per thread of the span kernels

template <bool IS_MAX>
static int pool_span_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, hipStream_t st)
{
    PoolShape s = make_shape(N, C, H, W, k, 1, kSpanR, H - (k - 1), W - (k - 1), 4);
    const dim3 grid((unsigned)(s.per_xcd * kPoolXcds)), block(kPoolThreads);
    if (k == 4) pool_span_fwd_kernel<4, kSpanR, IS_MAX><<<grid, block, 0, st>>>((const float *)x, (float *)y, am, s);
    else pool_span_fwd_kernel<8, kSpanR, IS_MAX><<<grid, block, 0, st>>>((const float *)x, (float *)y, am, s);
    return check_launch();
}

template <bool IS_MAX>
static int pool_span_bwd(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k, hipStream_t st)
{
    PoolShape s = make_shape(N, C, H, W, k, 1, kSpanR, H, W, 4);
    const dim3 grid((unsigned)(s.per_xcd * kPoolXcds)), block(kPoolThreads);
    if (k == 4) pool_span_bwd_kernel<4, kSpanR, IS_MAX><<<grid, block, 0, st>>>((const float *)dy, am, (float *)dx, s);
    else pool_span_bwd_kernel<8, kSpanR, IS_MAX><<<grid, block, 0, st>>>((const float *)dy, am, (float *)dx, s);
    return check_launch();
}

static bool pool_span_ok(int N, int C, int H, int W, int k, int d, size_t elem)
{
    return d == 1 && (k == 4 || k == 8) && elem == 4 && (long)N * C * ((H + kSpanR - 1) / kSpanR) * ((W + 255) / 256) < 0x7ffffff0L;
}

template <typename T, bool IS_MAX>
static int pool_fwd_dispatch(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                             hipStream_t st)
{
    if (pool_span_ok(N, C, H, W, k, d, sizeof(T))) return pool_span_fwd<IS_MAX>(x, y, am, N, C, H, W, k, st);
    // 2 x 2 and 3 x 3 windows: the walking kernels with 16-byte accesses -- unless the rows of an fp32 map begin at
    // odd multiples of 4 bytes (odd width), where a 16-byte access per lane is slower than four 4-byte ones
    if (pool_walk_ok(N, C, H, W, k, d, sizeof(T) == 4 ? DSK_F32 : DSK_BF16) && (sizeof(T) == 2 || W % 2 == 0))
        return launch_pool_walk_fwd(x, y, am, N, C, H, W, k, d, IS_MAX, sizeof(T) == 4 ? DSK_F32 : DSK_BF16, st);
    // pairs pay where the instruction count binds: 2-byte pixels (fp32 kernels run as fast with one pixel per thread)
    return pool_pairs(W, d) && sizeof(T) == 2 ? pool_fwd_dispatch<T, IS_MAX, 2>(x, y, am, N, C, H, W, k, d, st)
                            : pool_fwd_dispatch<T, IS_MAX, 1>(x, y, am, N, C, H, W, k, d, st);
}

template <typename T, bool IS_MAX>
static int pool_bwd_dispatch(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k,
                             int d, hipStream_t st)
{
    if (pool_span_ok(N, C, H, W, k, d, sizeof(T)) && (W - (k - 1)) % 4 == 0)
        return pool_span_bwd<IS_MAX>(dy, am, dx, N, C, H, W, k, st);
    if (pool_walk_ok(N, C, H, W, k, d, sizeof(T) == 4 ? DSK_F32 : DSK_BF16))
        return launch_pool_walk_bwd(dy, am, dx, nullptr, nullptr, DSK_ACT_NONE, nullptr, N, C, H, W, k, d, IS_MAX,
                                    sizeof(T) == 4 ? DSK_F32 : DSK_BF16, st);
    // ... and the max-pool gradient, which loads a tap index with every pixel
    return pool_pairs(W, d) && (sizeof(T) == 2 || IS_MAX) ? pool_bwd_dispatch<T, IS_MAX, 2>(dy, am, dx, N, C, H, W, k, d, st)
                            : pool_bwd_dispatch<T, IS_MAX, 1>(dy, am, dx, N, C, H, W, k, d, st);
}

int launch_maxpool_fwd(const void *x, void *y, uint8_t *am, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st)
{
    return t == DSK_F32 ? pool_fwd_dispatch<float, true>(x, y, am, N, C, H, W, k, d, st)
                        : pool_fwd_dispatch<bf16, true>(x, y, am, N, C, H, W, k, d, st);
}

int launch_maxpool_bwd(const void *dy, const uint8_t *am, void *dx, int N, int C, int H, int W, int k, int d,
                       dsk_dtype t, hipStream_t st)
{
    return t == DSK_F32 ? pool_bwd_dispatch<float, true>(dy, am, dx, N, C, H, W, k, d, st)
                        : pool_bwd_dispatch<bf16, true>(dy, am, dx, N, C, H, W, k, d, st);
}

int launch_avgpool_fwd(const void *x, void *y, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st)
{
    return t == DSK_F32 ? pool_fwd_dispatch<float, false>(x, y, nullptr, N, C, H, W, k, d, st)
                        : pool_fwd_dispatch<bf16, false>(x, y, nullptr, N, C, H, W, k, d, st);
}

int launch_avgpool_bwd(const void *dy, void *dx, int N, int C, int H, int W, int k, int d, dsk_dtype t,
                       hipStream_t st)
{
    return t == DSK_F32 ? pool_bwd_dispatch<float, false>(dy, nullptr, dx, N, C, H, W, k, d, st)
                        : pool_bwd_dispatch<bf16, false>(dy, nullptr, dx, N, C, H, W, k, d, st);
}

} // namespace dsk
