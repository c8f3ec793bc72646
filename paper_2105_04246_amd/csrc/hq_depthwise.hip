// Depthwise convolution (one R x S filter per channel) with the same fused epilogue as the
// GEMMs.  No matrix cores: per output there are only R*S multiply-accumulates against ~2
// bytes of traffic, so the layer is bound by memory, not arithmetic (the depthwise rows of
// the paper's Table 5).  Forward and input gradient are the same gather with the tap offsets
// mirrored; the weight gradient reduces over all pixels per (tap, channel).
#include "hq_device.h"
#include "hq_internal.h"

namespace {

struct DwArgs {
    const int8_t *A, *Wt;
    const int32_t *wsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int M, C;                      // output pixels, channels
    int R, S, Hs, Ws, Ho, Wo, stride, pad, dgrad;
    int sr_on;                     // 1: stochastic rounding with the seed below
    HqSr sr;
};

__device__ inline int sbyte(int v, int k) { return (v << (24 - 8 * k)) >> 24; }

// One thread: one output pixel, four consecutive channels (one 32-bit word of codes).
__global__ __launch_bounds__(HQ_THREADS) void hq_depthwise_kernel(const DwArgs a)
{
    __shared__ int red[4 * (HQ_THREADS / 64)];
    const int c4n = a.C >> 2;
    const size_t total = (size_t)a.M * c4n;
    const int za = a.aq->zero_point;
    const int fill = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const bool fused = a.out32 == nullptr;
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqRequant rq = {1.0f, 0.0f, 0.0f, 0};
    if (fused) rq = hq_make_requant(acc_scale, a.range->qp, a.range->qlo, a.range->qhi);
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;

    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % c4n) * 4;
        const int m = (int)(idx / c4n);
        const int x = m % a.Wo, y = (m / a.Wo) % a.Ho, b = m / (a.Wo * a.Ho);
        const int8_t *img = a.A + (size_t)b * a.Hs * a.Ws * a.C;
        const int y0 = a.dgrad ? y + a.pad : y * a.stride - a.pad;
        const int x0 = a.dgrad ? x + a.pad : x * a.stride - a.pad;
        int acc[4] = {0, 0, 0, 0};
        for (int r = 0; r < a.R; r++) {
            for (int s = 0; s < a.S; s++) {
                int iy, ix; bool ok = true;
                if (!a.dgrad) { iy = y0 + r; ix = x0 + s; }
                else {
                    iy = y0 - r; ix = x0 - s;
                    if (a.stride != 1) {
                        ok = iy >= 0 && ix >= 0 && (iy % a.stride == 0) && (ix % a.stride == 0);
                        iy /= a.stride; ix /= a.stride;
                    }
                }
                ok = ok && iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws;
                const int xv = ok ? *reinterpret_cast<const int *>(img + ((size_t)iy * a.Ws + ix) * a.C + c) : fill;
                const int wv = *reinterpret_cast<const int *>(a.Wt + (size_t)(r * a.S + s) * a.C + c);
#pragma unroll
                for (int e = 0; e < 4; e++) acc[e] += sbyte(xv, e) * sbyte(wv, e);
            }
        }
        const v4i ws = *reinterpret_cast<const v4i *>(a.wsum + c);
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int cv = acc[e] - za * ws[e];
            mn = min(mn, cv); mx = max(mx, cv);
            q[e] = cv;
        }
        if (fused) {
#pragma unroll
            for (int e = 0; e < 4; e++)
                q[e] = a.sr_on ? hq_requant_sr(q[e], rq, a.sr, (size_t)m * a.C + c + e, nlo, nhi) : hq_requant(q[e], rq, nlo, nhi);
            *reinterpret_cast<unsigned *>(a.out8 + (size_t)m * a.C + c) = hq_pack4(q[0], q[1], q[2], q[3]);
        } else {
            v4i v = {q[0], q[1], q[2], q[3]};
            *reinterpret_cast<v4i *>(a.out32 + (size_t)m * a.C + c) = v;
        }
    }
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.C);
        if (fused) *a.outq = a.range->qp;
    }
}

// ---------------------------------------------------------------------------------------
// 3x3, stride 1 (forward, and input gradient as the same stencil with mirrored taps): the
// shape of the depthwise layers of MobileNetV2-style blocks (Table 5, DW rows).
// A thread owns four channels of one output column and slides down a strip of rows, keeping
// the 3x3 window in registers as one word per (window row, channel) with the three horizontally
// adjacent values in its bytes (two v_perm_b32 per word), so that an output is three 4-way byte
// dot products (v_dot4) instead of nine multiply-adds on unpacked values.  Per output row the
// thread loads three new words (one input row of the window), so an input byte is requested 3 times (by the three neighbouring
// columns, which sit in adjacent lanes and hit the same cache lines) instead of 9.  Lanes run
// along (column, channel) of a row, which is how NHWC lies in memory: loads and the 4-code
// stores are contiguous across the wavefront.  The next row's words are requested before the
// current row is multiplied.
// ---------------------------------------------------------------------------------------
struct Dw3Args {
    const int8_t *A, *Wt;
    const int32_t *wsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int B, H, W, C;                // input and output have the same size (pad 1)
    int rows_per_strip, flip;
};

// Three packed words (four channels each of the pixels left, middle, right) -> four words, one per
// channel, holding that channel's three horizontally adjacent values and a zero byte: the operand
// of a 4-way byte dot product against the three taps of a filter row.
__device__ inline void dw_transpose3(int l, int m, int r, int *t)
{
#pragma unroll
    for (int e = 0; e < 4; e++) {
        // v_perm_b32: selector bytes 0..3 pick bytes of the second source, 4..7 of the first, 0x0c is zero
        const unsigned lm = __builtin_amdgcn_perm((unsigned)m, (unsigned)l, 0x0c0c0000u | (unsigned)e | ((4u + e) << 8));
        t[e] = (int)__builtin_amdgcn_perm((unsigned)r, lm, 0x0c000100u | ((4u + e) << 16));
    }
}

__global__ __launch_bounds__(HQ_THREADS) void hq_dw3x3_kernel(const Dw3Args a)
{
    __shared__ int red[4 * (HQ_THREADS / 64)];
    const int c4n = a.C >> 2, rowwords = a.W * c4n;
    const int q = blockIdx.x * HQ_THREADS + threadIdx.x;           // word inside an output row
    const bool live = q < rowwords;
    const int qq = live ? q : 0;
    const int ox = qq / c4n, c = (qq - ox * c4n) * 4;
    const int y0 = blockIdx.y * a.rows_per_strip, y1 = min(a.H, y0 + a.rows_per_strip);
    const int8_t *img = a.A + (size_t)blockIdx.z * a.H * a.W * a.C;
    const size_t out_img = (size_t)blockIdx.z * a.H * a.W;

    const int za = a.aq->zero_point;
    const int fill = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const bool fused = a.out32 == nullptr;
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (fused) ep = hq_make_epilogue(acc_scale, a.range);

    // weights of the four channels: per filter row and channel one word (w[r][0], w[r][1], w[r][2], 0);
    // mirrored for the input gradient
    int wt[3][4];
#pragma unroll
    for (int r = 0; r < 3; r++) {
        int pk[3];
#pragma unroll
        for (int sx = 0; sx < 3; sx++) {
            const int t = r * 3 + sx, ts = a.flip ? 8 - t : t;
            pk[sx] = *reinterpret_cast<const int *>(a.Wt + (size_t)ts * a.C + c);
        }
        dw_transpose3(pk[0], pk[1], pk[2], wt[r]);
    }
    const v4i wsv = *reinterpret_cast<const v4i *>(a.wsum + c);
    int zw[4];
#pragma unroll
    for (int e = 0; e < 4; e++) zw[e] = za * wsv[e];

    const bool okl = ox > 0, okr = ox + 1 < a.W;
    const size_t rowbytes = (size_t)a.W * a.C;
    const int8_t *pcol = img + (size_t)ox * a.C + c;                 // this thread's column in input row 0
    auto load_row = [&](const int8_t *p, bool rowok, int *dst) {      // three packed words of one input row
        dst[0] = (rowok && okl) ? *reinterpret_cast<const int *>(p - a.C) : fill;
        dst[1] = rowok ? *reinterpret_cast<const int *>(p) : fill;
        dst[2] = (rowok && okr) ? *reinterpret_cast<const int *>(p + a.C) : fill;
    };
    const int8_t *pn = pcol + (size_t)(y0 > 0 ? y0 - 1 : 0) * rowbytes;   // walks down the input rows
    size_t o = (out_img + (size_t)y0 * a.W + ox) * a.C + c;           // output word of row oy, advanced per row

    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;
    int win[3][4];                                                   // [row slot][channel]: (left, middle, right, 0)
    int ring[3][3];                                                  // packed words of the next three input rows
    if (live) {
        int tmp[3];
        load_row(pn, y0 > 0, tmp);                                   // row y0 - 1
        if (y0 > 0) pn += rowbytes;
        dw_transpose3(tmp[0], tmp[1], tmp[2], win[0]);
        load_row(pn, true, tmp);                                     // row y0
        pn += rowbytes;
        dw_transpose3(tmp[0], tmp[1], tmp[2], win[1]);
#pragma unroll
        for (int k = 0; k < 3; k++) {                                // rows y0 + 1 .. y0 + 3 in flight
            load_row(pn, y0 + 1 + k < a.H, ring[k]);
            pn += rowbytes;
        }
    }
    // one output row; TOP / MID / BOT name the register slots of input rows oy-1, oy, oy+1
#define DW_STEP(TOP, MID, BOT, RING)                                                                        \
    if (live && oy < y1) {                                                                            \
        dw_transpose3(ring[RING][0], ring[RING][1], ring[RING][2], win[BOT]);                           \
        if (oy + 3 < y1) { load_row(pn, oy + 4 < a.H, ring[RING]); pn += rowbytes; }                   \
        int cv[4];                                                                                    \
        _Pragma("unroll") for (int e = 0; e < 4; e++) {                                                 \
            int acc = __builtin_amdgcn_sdot4(win[TOP][e], wt[0][e], -zw[e], false);                   \
            acc = __builtin_amdgcn_sdot4(win[MID][e], wt[1][e], acc, false);                          \
            cv[e] = __builtin_amdgcn_sdot4(win[BOT][e], wt[2][e], acc, false);                        \
        }                                                                                             \
        if (fused) {                                                                                  \
            int wd;                                                                                   \
            if (ep.full_grid) hq_requant_group<4, true>(cv, ep, mn, mx, nlo, nhi, &wd);               \
            else hq_requant_group<4, false>(cv, ep, mn, mx, nlo, nhi, &wd);                            \
            *reinterpret_cast<int *>(a.out8 + o) = wd;                                                \
        } else {                                                                                      \
            hq_minmax_group<4>(cv, mn, mx);                                                           \
            const v4i v = {cv[0], cv[1], cv[2], cv[3]};                                               \
            *reinterpret_cast<v4i *>(a.out32 + o) = v;                                                \
        }                                                                                             \
    }                                                                                                 \
    oy++; o += rowbytes;
    for (int oy = y0; oy < y1;) {
        DW_STEP(0, 1, 2, 0)
        DW_STEP(1, 2, 0, 1)
        DW_STEP(2, 0, 1, 2)
    }
#undef DW_STEP
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.B * a.H * a.W * (unsigned long long)a.C);
        if (fused) *a.outq = a.range->qp;
    }
}

// Weight gradient: acc[tap][c] = sum_m Xg[m][tap][c] * G[m][c], plus the column sums that
// remove the zero points.  Each workgroup takes a run of pixels; a thread owns four channels
// and strides over the run; partial sums meet in LDS and leave with one atomic per value.
constexpr int DW_MAX_TAPS = 9;

struct DwWgradArgs {
    const int8_t *X, *G;
    const hq_qparams *xq;
    int32_t *acc, *gsum, *xsum;
    int M, C, R, S, H, W, OH, OW, stride, pad;
    int m_per_block;
    int CT;                        // channels per workgroup (multiple of 4, <= 256)
};

__global__ __launch_bounds__(HQ_THREADS) void hq_depthwise_wgrad_kernel(const DwWgradArgs a)
{
    extern __shared__ int lds[];                 // [taps][CT] acc, [CT] gsum, [taps][CT] xsum
    const int taps = a.R * a.S, CT = a.CT;
    const int ct0 = blockIdx.y * CT, ct = min(CT, a.C - ct0);      // this workgroup's channel tile
    const int words = (2 * taps + 1) * CT;
    for (int i = threadIdx.x; i < words; i += blockDim.x) lds[i] = 0;
    __syncthreads();
    const int zx = a.xq->zero_point;
    const int fill = (int)((unsigned)(zx & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const int lanes_per_pixel = ct >> 2;                           // <= 64
    const int pixels_per_pass = HQ_THREADS / lanes_per_pixel;
    const int cg = threadIdx.x % lanes_per_pixel, prow = threadIdx.x / lanes_per_pixel;
    const int cl = cg * 4, c = ct0 + cl;
    const int m_begin = blockIdx.x * a.m_per_block, m_end = min(a.M, m_begin + a.m_per_block);
    if (prow < pixels_per_pass) {
        int acc[DW_MAX_TAPS][4], xs[DW_MAX_TAPS][4], gs[4] = {0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < DW_MAX_TAPS; t++)
#pragma unroll
            for (int e = 0; e < 4; e++) { acc[t][e] = 0; xs[t][e] = 0; }
        for (int m = m_begin + prow; m < m_end; m += pixels_per_pass) {
            const int ow = m % a.OW, oh = (m / a.OW) % a.OH, b = m / (a.OW * a.OH);
            const int gv = *reinterpret_cast<const int *>(a.G + (size_t)m * a.C + c);
            int g[4];
#pragma unroll
            for (int e = 0; e < 4; e++) { g[e] = sbyte(gv, e); gs[e] += g[e]; }
#pragma unroll
            for (int t = 0; t < DW_MAX_TAPS; t++) {
                if (t < taps) {
                    const int r = t / a.S, s = t % a.S;
                    const int iy = oh * a.stride - a.pad + r, ix = ow * a.stride - a.pad + s;
                    const bool ok = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                    const int xv = ok ? *reinterpret_cast<const int *>(a.X + (((size_t)b * a.H + iy) * a.W + ix) * a.C + c) : fill;
#pragma unroll
                    for (int e = 0; e < 4; e++) { const int x = sbyte(xv, e); acc[t][e] += x * g[e]; xs[t][e] += x; }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < DW_MAX_TAPS; t++)
            if (t < taps)
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    atomicAdd(&lds[t * CT + cl + e], acc[t][e]);
                    atomicAdd(&lds[(taps + 1 + t) * CT + cl + e], xs[t][e]);
                }
#pragma unroll
        for (int e = 0; e < 4; e++) atomicAdd(&lds[taps * CT + cl + e], gs[e]);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < words; i += blockDim.x) {
        const int v = lds[i];
        const int row = i / CT, col = i % CT;
        if (v == 0 || col >= ct) continue;
        if (row < taps) atomicAdd(a.acc + row * a.C + ct0 + col, v);
        else if (row == taps) atomicAdd(a.gsum + ct0 + col, v);
        else atomicAdd(a.xsum + (row - taps - 1) * a.C + ct0 + col, v);
    }
}

// 3x3, stride 1, pad 1 weight gradient: the thread layout of hq_dw3x3_kernel (four channels of
// one column, sliding down a strip of rows), four output rows at a time.  The reduction runs over
// pixels, so the rows are byte-transposed: four packed words (four rows, four channels each)
// become four words holding four vertically adjacent values of one channel (eight v_perm_b32),
// and a tap's contribution of the four rows is one 4-way dot product against the transposed
// gradient word.  The three row taps are the transposed block shifted by one row either way
// (v_alignbyte with the neighbouring blocks).  A workgroup walks over several images and keeps
// its 36 sums per thread in registers; threads that share channels meet in LDS, and the workgroup
// leaves with one atomic per value.  The column sums of the input that remove the gradient's
// zero point are only gathered when that zero point is not 0.
struct Dw3WgradArgs {
    const int8_t *X, *G;
    const hq_qparams *xq, *gq;
    int32_t *acc, *gsum, *xsum;
    int B, H, W, C;
    int rows_per_strip;            // multiple of 4
};

// four words = four rows of four channels -> t[e] = (row0[e], row1[e], row2[e], row3[e])
__device__ inline void dw_transpose4(int a0, int a1, int a2, int a3, int *t)
{
    const unsigned p0 = __builtin_amdgcn_perm((unsigned)a1, (unsigned)a0, 0x05010400u);   // (a0.0, a1.0, a0.1, a1.1)
    const unsigned p1 = __builtin_amdgcn_perm((unsigned)a1, (unsigned)a0, 0x07030602u);   // (a0.2, a1.2, a0.3, a1.3)
    const unsigned q0 = __builtin_amdgcn_perm((unsigned)a3, (unsigned)a2, 0x05010400u);
    const unsigned q1 = __builtin_amdgcn_perm((unsigned)a3, (unsigned)a2, 0x07030602u);
    t[0] = (int)__builtin_amdgcn_perm(q0, p0, 0x05040100u);
    t[1] = (int)__builtin_amdgcn_perm(q0, p0, 0x07060302u);
    t[2] = (int)__builtin_amdgcn_perm(q1, p1, 0x05040100u);
    t[3] = (int)__builtin_amdgcn_perm(q1, p1, 0x07060302u);
}

__global__ __launch_bounds__(HQ_THREADS) void hq_dw3x3_wgrad_kernel(const Dw3WgradArgs a)
{
    extern __shared__ int lds[];                 // [9][C] acc, [C] gsum, [9][C] xsum
    const int words = 19 * a.C;
    for (int i = threadIdx.x; i < words; i += HQ_THREADS) lds[i] = 0;
    __syncthreads();
    const int c4n = a.C >> 2, rowwords = a.W * c4n;
    const int q = blockIdx.x * HQ_THREADS + threadIdx.x;
    const bool live = q < rowwords;
    const int qq = live ? q : 0;
    const int ox = qq / c4n, c = (qq - ox * c4n) * 4;
    const int y0 = blockIdx.y * a.rows_per_strip, y1 = min(a.H, y0 + a.rows_per_strip);
    const int zx = a.xq->zero_point;
    const bool want_xsum = a.gq->zero_point != 0;
    const int fill = (int)((unsigned)(zx & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const bool okl = ox > 0, okr = ox + 1 < a.W;
    const size_t rowbytes = (size_t)a.W * a.C;

    int acc[9][4], xs[9][4], gs[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 9; t++)
#pragma unroll
        for (int e = 0; e < 4; e++) { acc[t][e] = 0; xs[t][e] = 0; }

    if (live && y0 < y1) {
        for (int b = blockIdx.z; b < a.B; b += gridDim.z) {
            const int8_t *ximg = a.X + (size_t)b * a.H * rowbytes + (size_t)ox * a.C + c;
            const int8_t *gimg = a.G + (size_t)b * a.H * rowbytes + (size_t)ox * a.C + c;
            // block of four input rows starting at row y: raw[row][column], zero-point code outside the image
            auto load_x = [&](int y, int (&raw)[4][3]) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const int iy = y + k;
                    const bool rok = iy >= 0 && iy < a.H;
                    const int8_t *p = ximg + (ptrdiff_t)iy * rowbytes;
                    const int l = *reinterpret_cast<const int *>(rok && okl ? p - a.C : ximg);
                    const int m = *reinterpret_cast<const int *>(rok ? p : ximg);
                    const int r = *reinterpret_cast<const int *>(rok && okr ? p + a.C : ximg);
                    raw[k][0] = rok && okl ? l : fill; raw[k][1] = rok ? m : fill; raw[k][2] = rok && okr ? r : fill;
                }
            };
            // gradient rows y .. y+3 of this column; rows past the strip count as zero
            auto load_g = [&](int y, int (&raw)[4]) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const bool rok = y + k < y1;
                    const int v = *reinterpret_cast<const int *>(rok ? gimg + (size_t)(y + k) * rowbytes : gimg);
                    raw[k] = rok ? v : 0;
                }
            };
            auto transpose_x = [&](const int (&raw)[4][3], int (&t)[3][4]) {
#pragma unroll
                for (int sx = 0; sx < 3; sx++) dw_transpose4(raw[0][sx], raw[1][sx], raw[2][sx], raw[3][sx], t[sx]);
            };
            int prev[3][4], cur[3][4], nxt[3][4];             // [column][channel]: four rows in the bytes
            int xraw[4][3], graw[4];
            {
                // of the block above the strip only its last row (y0 - 1) is ever read
                const int iy = y0 - 1;
                const bool rok = iy >= 0;
                const int8_t *p = ximg + (ptrdiff_t)iy * rowbytes;
                const int l = *reinterpret_cast<const int *>(rok && okl ? p - a.C : ximg);
                const int m = *reinterpret_cast<const int *>(rok ? p : ximg);
                const int r = *reinterpret_cast<const int *>(rok && okr ? p + a.C : ximg);
                const int row3[3] = {rok && okl ? l : fill, rok ? m : fill, rok && okr ? r : fill};
#pragma unroll
                for (int sx = 0; sx < 3; sx++) dw_transpose4(0, 0, 0, row3[sx], prev[sx]);
            }
            load_x(y0, xraw); transpose_x(xraw, cur);
            load_x(y0 + 4, xraw);                                // in flight: rows y0+4 .. y0+7, gradient rows y0 .. y0+3
            load_g(y0, graw);
            for (int oy = y0; oy < y1; oy += 4) {
                transpose_x(xraw, nxt);
                int gt[4];
                dw_transpose4(graw[0], graw[1], graw[2], graw[3], gt);
                if (oy + 4 < y1) { load_x(oy + 8, xraw); load_g(oy + 4, graw); }
                // rows of this block that exist as output rows: a byte of ones per row (input column sums)
                const int nrow = min(4, y1 - oy);
                const int ones = nrow >= 4 ? 0x01010101 : nrow == 3 ? 0x00010101 : nrow == 2 ? 0x00000101 : 0x00000001;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    gs[e] = __builtin_amdgcn_sdot4(gt[e], 0x01010101, gs[e], false);
#pragma unroll
                    for (int sx = 0; sx < 3; sx++) {
                        const int top = (int)__builtin_amdgcn_alignbyte((unsigned)cur[sx][e], (unsigned)prev[sx][e], 3);   // rows oy-1 .. oy+2
                        const int bot = (int)__builtin_amdgcn_alignbyte((unsigned)nxt[sx][e], (unsigned)cur[sx][e], 1);    // rows oy+1 .. oy+4
                        acc[sx][e] = __builtin_amdgcn_sdot4(top, gt[e], acc[sx][e], false);
                        acc[3 + sx][e] = __builtin_amdgcn_sdot4(cur[sx][e], gt[e], acc[3 + sx][e], false);
                        acc[6 + sx][e] = __builtin_amdgcn_sdot4(bot, gt[e], acc[6 + sx][e], false);
                        if (want_xsum) {
                            xs[sx][e] = __builtin_amdgcn_sdot4(top, ones, xs[sx][e], false);
                            xs[3 + sx][e] = __builtin_amdgcn_sdot4(cur[sx][e], ones, xs[3 + sx][e], false);
                            xs[6 + sx][e] = __builtin_amdgcn_sdot4(bot, ones, xs[6 + sx][e], false);
                        }
                    }
                }
#pragma unroll
                for (int sx = 0; sx < 3; sx++)
#pragma unroll
                    for (int e = 0; e < 4; e++) { prev[sx][e] = cur[sx][e]; cur[sx][e] = nxt[sx][e]; }
            }
        }
#pragma unroll
        for (int t = 0; t < 9; t++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
                atomicAdd(&lds[t * a.C + c + e], acc[t][e]);
                if (want_xsum) atomicAdd(&lds[(10 + t) * a.C + c + e], xs[t][e]);
            }
#pragma unroll
        for (int e = 0; e < 4; e++) atomicAdd(&lds[9 * a.C + c + e], gs[e]);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < words; i += HQ_THREADS) {
        const int v = lds[i];
        if (v == 0) continue;
        const int row = i / a.C, col = i - row * a.C;
        if (row < 9) atomicAdd(a.acc + row * a.C + col, v);
        else if (row == 9) atomicAdd(a.gsum + col, v);
        else atomicAdd(a.xsum + (row - 10) * a.C + col, v);
    }
}

__global__ void dw_zero_kernel(int32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

__global__ void dw_wgrad_finalize_kernel(const int32_t *acc, const int32_t *gsum, const int32_t *xsum,
                                         const hq_qparams *xq, const hq_qparams *gq, unsigned M, int K, int C,
                                         float *dW, int32_t *dW_acc, const HqRideAlong ride)
{
    if (hq_ride_along(ride)) return;
    const unsigned zx = (unsigned)xq->zero_point, zg = (unsigned)gq->zero_point;
    const float s = __fmul_rn(xq->scale, gq->scale);
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const unsigned c = (unsigned)acc[k] - zx * (unsigned)gsum[k % C] - zg * (unsigned)xsum[k] + M * zx * zg;
    if (dW_acc) dW_acc[k] = (int)c;
    dW[k] = __fmul_rn(s, (float)(int)c);
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

} // namespace

int hq_launch_depthwise(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Wt,
                        const hq_qparams *bq, const int32_t *wsum, const hq_range *range, int8_t *out8,
                        int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed)
{
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    if (sr_seed && out32) return HQ_E_BADARG;
    DwArgs a;
    a.sr_on = sr_seed ? 1 : 0;
    a.sr.k0 = sr_seed ? (unsigned)*sr_seed : 0u; a.sr.k1 = sr_seed ? (unsigned)(*sr_seed >> 32) : 0u;
    a.A = A; a.Wt = Wt; a.wsum = wsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.C = p->C; a.R = p->R; a.S = p->S; a.stride = p->stride; a.pad = p->pad; a.dgrad = dgrad;
    if (!dgrad) { a.M = p->B * OH * OW; a.Hs = p->H; a.Ws = p->W; a.Ho = OH; a.Wo = OW; }
    else        { a.M = p->B * p->H * p->W; a.Hs = OH; a.Ws = OW; a.Ho = p->H; a.Wo = p->W; }
    if (!sr_seed && p->R == 3 && p->S == 3 && p->stride == 1 && p->pad == 1 && p->B <= 65535) {
        Dw3Args d;
        d.A = A; d.Wt = Wt; d.wsum = wsum; d.aq = aq; d.bq = bq; d.range = range;
        d.out8 = out8; d.out32 = out32; d.outq = outq; d.st = st;
        d.B = p->B; d.H = p->H; d.W = p->W; d.C = p->C; d.flip = dgrad;
        const int xb = (p->W * (p->C / 4) + HQ_THREADS - 1) / HQ_THREADS;
        // strips: enough workgroups to fill the chip several times, rows per strip a multiple of 3
        int strips = (4096 + xb * p->B - 1) / (xb * p->B);
        if (strips < 1) strips = 1;
        int rps = (p->H + strips - 1) / strips;
        rps = (rps + 2) / 3 * 3;
        if (rps < 6) rps = 6;
        d.rows_per_strip = rps;
        strips = (p->H + rps - 1) / rps;
        hipLaunchKernelGGL(hq_dw3x3_kernel, dim3((unsigned)xb, (unsigned)strips, (unsigned)p->B), dim3(HQ_THREADS), 0,
                           stream, d);
        return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
    }
    const size_t total = (size_t)a.M * (a.C / 4);
    size_t blocks = (total + HQ_THREADS - 1) / HQ_THREADS;
    if (blocks > 256u * 64u) blocks = 256u * 64u;
    hipLaunchKernelGGL(hq_depthwise_kernel, dim3((unsigned)blocks), dim3(HQ_THREADS), 0, stream, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

int hq_launch_depthwise_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                              const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, hipStream_t stream,
                              const HqRideAlong *ride)
{
    if (p->R * p->S > DW_MAX_TAPS) return HQ_E_BADSHAPE;
    HqRideAlong ra = {nullptr, nullptr, 0, 0};
    if (ride) ra = *ride;
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    const int taps = p->R * p->S;
    const size_t K = (size_t)taps * p->C;
    DwWgradArgs a;
    a.X = X; a.G = dY; a.xq = xq;
    char *w = static_cast<char *>(ws);
    a.acc = reinterpret_cast<int32_t *>(w);
    a.gsum = reinterpret_cast<int32_t *>(w + align16(4 * K));
    a.xsum = reinterpret_cast<int32_t *>(w + align16(4 * K) + align16(4 * (size_t)p->C));
    a.M = p->B * OH * OW; a.C = p->C; a.R = p->R; a.S = p->S; a.H = p->H; a.W = p->W; a.OH = OH; a.OW = OW;
    a.stride = p->stride; a.pad = p->pad;
    const size_t ws_words = hq_wgrad_workspace_bytes(p) / 4;
    hipLaunchKernelGGL(dw_zero_kernel, dim3(16), dim3(256), 0, stream, a.acc, ws_words);
    if (p->R == 3 && p->S == 3 && p->stride == 1 && p->pad == 1 && 19 * (size_t)p->C * 4 <= 64 * 1024) {
        Dw3WgradArgs d;
        d.X = X; d.G = dY; d.xq = xq; d.gq = gq; d.acc = a.acc; d.gsum = a.gsum; d.xsum = a.xsum;
        d.B = p->B; d.H = p->H; d.W = p->W; d.C = p->C;
        const int xb = (p->W * (p->C / 4) + HQ_THREADS - 1) / HQ_THREADS;
        // about four workgroups per compute unit: strips of at least 16 rows (a strip also reads the row
        // above it and up to four rows below), then images in turn
        int strips = p->H / 16 > 0 ? p->H / 16 : 1;
        while (strips > 1 && xb * strips > 1024) strips--;
        int rps = (p->H + strips - 1) / strips;
        rps = (rps + 3) / 4 * 4;
        d.rows_per_strip = rps;
        strips = (p->H + rps - 1) / rps;
        int gz = 768 / (xb * strips);
        if (gz < 1) gz = 1;
        if (gz > p->B) gz = p->B;
        hipLaunchKernelGGL(hq_dw3x3_wgrad_kernel, dim3((unsigned)xb, (unsigned)strips, (unsigned)gz), dim3(HQ_THREADS),
                           19 * (size_t)p->C * 4, stream, d);
        ra.first = (int)((K + 255) / 256);
        hipLaunchKernelGGL(dw_wgrad_finalize_kernel, dim3((unsigned)((K + 255) / 256) + (unsigned)ra.n), dim3(256), 0, stream,
                           a.acc, a.gsum, a.xsum, xq, gq, (unsigned)a.M, (int)K, p->C, dW, dW_acc, ra);
        return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
    }
    a.CT = p->C < 256 ? p->C : 256;
    const int ctiles = (p->C + a.CT - 1) / a.CT;
    int blocks = (2048 + ctiles - 1) / ctiles;
    a.m_per_block = (a.M + blocks - 1) / blocks;
    if (a.m_per_block < 1) a.m_per_block = 1;
    blocks = (a.M + a.m_per_block - 1) / a.m_per_block;
    const size_t lds_bytes = (size_t)(2 * taps + 1) * a.CT * 4;       // at most 19 KiB
    hipLaunchKernelGGL(hq_depthwise_wgrad_kernel, dim3((unsigned)blocks, (unsigned)ctiles), dim3(HQ_THREADS),
                       lds_bytes, stream, a);
    ra.first = (int)((K + 255) / 256);
    hipLaunchKernelGGL(dw_wgrad_finalize_kernel, dim3((unsigned)((K + 255) / 256) + (unsigned)ra.n), dim3(256), 0, stream,
                       a.acc, a.gsum, a.xsum, xq, gq, (unsigned)a.M, (int)K, p->C, dW, dW_acc, ra);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}
