// Weight gradient G_W = X~^T . G~_Y on int8 MFMA (paper Sec. 3.1; kept in FP32, no quantizer).
//
//   acc[n][tap][c] = sum_m  G[m][n] * Xg[m][tap][c]          m = (b, oh, ow) over all output pixels
//
// The reduction runs over pixels, which is the slow dimension of both NHWC operands, while
// an MFMA lane wants 16 reduction-contiguous bytes.  Both tiles are therefore staged in LDS
// as they lie in memory ([pixel][channel], 16-byte coalesced loads) and read back through the
// transposing LDS load of gfx950 (ds_read_b64_tr_b8): 16 lanes hand in 16 row addresses and
// receive, per lane, one channel of 8 consecutive pixels.
//
// Zero points: taps outside the image are filled with X's zero-point code, rows past the end
// of the tensor with code 0 in both operands, and the raw sum is corrected afterwards by
//   c = acc - z_x * sum_m G[m][n] - z_g * sum_m Xg[m][tap][c] + M * z_x * z_g .
// The two column sums come from the same fragments (dot4 against ones) in the workgroups of
// the first tile column / row.  The pixel range is split over workgroups (split-K); partial
// tiles are merged with 32-bit integer atomics, which is exact in any order.
#include "hq_device.h"
#include "hq_internal.h"

namespace {

typedef __attribute__((__vector_size__(2 * sizeof(int)))) int tr_v2i;
#define LDS_PTR(T) __attribute__((address_space(3))) T *

constexpr int MB = 64;             // pixels staged per step (two MFMA k-steps of 32)

struct WgradArgs {
    const int8_t *X, *G;
    const hq_qparams *xq, *gq;
    int32_t *acc;                  // [N][taps][C], zeroed
    int32_t *gsum;                 // [N], zeroed
    int32_t *xsum;                 // [taps][C], zeroed
    int M, N, C;
    int R, S, H, W, OH, OW, stride, pad;
    int m_per_split;               // multiple of MB
    int ctiles;                    // tiles along C inside one tap
    int xt, yt, splits;            // tile columns (taps * ctiles), tile rows, pixel splits
    int g16, x16;                  // rows of G / X are 16-byte aligned (N % 16 == 0 / C % 16 == 0)
    int direct;                    // splits == 1: every sum has one writer, plain stores into acc (not zeroed)
    unsigned magic_OW, magic_OH;   // ceil(2^32 / d) for the pixel decode, or 0, 0 with magic_ok == 0: plain division
    int magic_ok;
};

__device__ inline v4i load16(const int8_t *p, int nbytes, bool aligned16)
{
    if (aligned16) return *reinterpret_cast<const v4i *>(p);
    v4i v;
    const int *q = reinterpret_cast<const int *>(p);
    v[0] = nbytes > 0 ? q[0] : 0;
    v[1] = nbytes > 4 ? q[1] : 0;
    v[2] = nbytes > 8 ? q[2] : 0;
    v[3] = nbytes > 12 ? q[3] : 0;
    return v;
}

// Fragment of one 32-channel x 32-pixel operand block for the 32x32x32 MFMA: lane l gets
// channel (l % 32) and the 16 pixels of half (l / 32).  `tile` points at row 0 of the k-step
// and column 0 of the 32-channel block.
template <int P> __device__ inline v4i read_frag_tr(const int8_t *tile, int lane)
{
    const int j = lane & 15, grp = (lane >> 4) & 1, half = lane >> 5;
    const int8_t *p = tile + (half * 16 + (j >> 1)) * P + 16 * grp + 8 * (j & 1);
    tr_v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(p));
    tr_v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(p + 8 * P));
    v4i f = {lo[0], lo[1], hi[0], hi[1]};
    return f;
}

// PACKED: layers with fewer than 16 input channels (a network's first layer).  The tile's columns
// then run over (tap, channel) pairs as they lie in a row of G_W, so a 16-byte chunk of the staged
// tile holds 16 / C taps (one 4-byte load each) instead of one tap padded with zeros.
// PACKED3: 3-channel inputs (RGB images).  The S * 3 <= 32 bytes of a filter row are contiguous in the
// input; every filter row gets 32 tile columns of its own (column = 32 * r + 3 * s + channel, the columns
// past S * 3 stay zero), so a thread's 16-byte chunk is 16 consecutive bytes of memory at any byte
// address: aligned loads plus a byte-wise funnel shift, then byte masks that replace the taps outside the
// image with the zero-point code.
template <int TN, int TK, bool PACKED, bool PACKED3 = false>
__global__ __launch_bounds__(HQ_THREADS) void hq_wgrad_kernel(const WgradArgs a)
{
    static_assert(!PACKED3 || PACKED, "the 3-channel form is a packed form");
    constexpr int PG = TN + 32, PX = TK + 32;           // LDS pitches (32 mod 64: best for the transposing reads)
    constexpr int WTN = TN / 2, WTK = TK / 2;           // 2 x 2 wavefronts
    constexpr int NT = WTN / 32, KT = WTK / 32;
    constexpr int GCH = TN / 16, XCH = TK / 16;         // 16-byte chunks per tile row
    constexpr int GLD = MB * GCH / HQ_THREADS, XLD = MB * XCH / HQ_THREADS;
    static_assert(GLD >= 1 && XLD >= 1, "tile too small for 256 loader threads");

    __shared__ __attribute__((aligned(16))) int8_t Gs[2][MB * PG];
    __shared__ __attribute__((aligned(16))) int8_t Xs[2][MB * PX];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: branches on it are uniform
    const int wn = wave >> 1, wk = wave & 1;
    // Workgroup -> (tile column bx, tile row by, pixel split bz).  All tile columns and rows of
    // one pixel split read the same X / dY rows; consecutive workgroup ids go round-robin over
    // the 8 XCDs, so the ids are re-mapped to keep one split's tiles on one XCD, back to back,
    // where its L2 serves the re-reads.
    int bx, by, bz;
    {
        const int per_split = a.xt * a.yt, total = per_split * a.splits;
        const int full = (total / (8 * per_split)) * (8 * per_split);   // ids covered by complete groups of 8 splits
        int split, tile;
        if ((int)blockIdx.x < full) {
            const int grp = blockIdx.x / (8 * per_split), r = blockIdx.x % (8 * per_split);
            split = grp * 8 + (r & 7); tile = r >> 3;
        } else {
            const int r = blockIdx.x - full;
            split = full / per_split + r / per_split; tile = r % per_split;
        }
        bx = tile % a.xt; by = tile / a.xt; bz = split;
    }
    const int tap = PACKED ? 0 : bx / a.ctiles, c0 = PACKED ? bx * TK : (bx % a.ctiles) * TK;
    const int tr = tap / a.S, ts = tap % a.S;
    const int kcols = a.R * a.S * a.C;            // PACKED: columns of the whole weight row
    const int n0 = by * TN;
    const int m_begin = bz * a.m_per_split;
    const int m_end = min(a.M, m_begin + a.m_per_split);
    const int zx = a.xq->zero_point;
    const int fill = (int)((unsigned)(zx & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    // (a column sum is only ever multiplied by the other operand's zero point: not formed when that is 0)
    const bool do_gsum = bx == 0 && wk == 0 && zx != 0;                      // column sums of G: first tile column
    const bool do_xsum = by == 0 && wn == 0 && a.gq->zero_point != 0;        // column sums of Xg: first tile row

    int pk_r[4], pk_s[4], pk_off[4], pk_ow[XLD], pk_oh[XLD], pk_b[XLD];
    if (PACKED) {
#pragma unroll
        for (int d = 0; d < 4; d++) {
            const int kc = c0 + (tid % XCH) * 16 + 4 * d;
            if (PACKED3) {
                // word d = bytes 4 * d .. 4 * d + 3 of this thread's 16 bytes of filter row pk_r[0]
                const int q = (c0 >> 4) + (tid % XCH);                 // 16-byte chunk: filter row q / 2, half q % 2
                pk_r[d] = (q >> 1) < a.R ? (q >> 1) : -1;
                pk_s[d] = 16 * (q & 1) + 4 * d;                        // first byte of the word inside the filter row
                pk_off[d] = pk_r[d] * a.W * 3 + 16 * (q & 1);
                continue;
            }
            const int t = kc / a.C, cc = kc - t * a.C;
            pk_r[d] = kc < kcols ? t / a.S : -1;
            pk_s[d] = t % a.S;
            pk_off[d] = (pk_r[d] * a.W + pk_s[d]) * a.C + cc;
        }
#pragma unroll
        for (int i = 0; i < XLD; i++) {
            const int m = m_begin + (tid + i * HQ_THREADS) / XCH;
            pk_ow[i] = m % a.OW; pk_oh[i] = (m / a.OW) % a.OH; pk_b[i] = m / (a.OW * a.OH);
        }
    }
    v4i greg[GLD], xreg[XLD];
    auto load_stage = [&](int mb) {
#pragma unroll
        for (int i = 0; i < GLD; i++) {
            const int idx = tid + i * HQ_THREADS, row = idx / GCH, col = (idx % GCH) * 16;
            const int m = mb + row, n = n0 + col;
            v4i v = {0, 0, 0, 0};
            if (m < m_end && n < a.N) v = load16(a.G + (size_t)m * a.N + n, a.N - n, a.g16);
            greg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < XLD; i++) {
            const int idx = tid + i * HQ_THREADS, row = idx / XCH, col = (idx % XCH) * 16;
            const int m = mb + row, c = c0 + col;
            v4i v = {0, 0, 0, 0};
            if (PACKED) {
                // the thread's four (tap, channel) columns never change; its pixels advance by MB per stage
                if (PACKED3 && m < m_end) {
                    const int iy0 = pk_oh[i] * a.stride - a.pad, ix0 = pk_ow[i] * a.stride - a.pad;
                    const int iy = iy0 + pk_r[0];
                    const bool rok = pk_r[0] >= 0 && iy >= 0 && iy < a.H;
                    const int8_t *base = a.X + (((ptrdiff_t)pk_b[i] * a.H + iy0) * a.W + ix0) * 3;
                    const int8_t *xend = a.X + (size_t)(a.M / (a.OH * a.OW)) * a.H * a.W * 3;
                    const int j0 = 3 * max(0, -ix0), j1 = 3 * min(a.S, a.W - ix0);   // bytes of a filter row inside the image
                    const v4i x = hq_load16_any(rok ? base + pk_off[0] : a.X, a.X, xend);
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        const unsigned mk = rok ? hq_bytemask(j0 - pk_s[d], j1 - pk_s[d]) : 0u;
                        const unsigned all = pk_r[0] >= 0 ? hq_bytemask(0, a.S * 3 - pk_s[d]) : 0u;   // columns that exist
                        v[d] = (int)(((unsigned)x[d] & mk) | ((unsigned)fill & all & ~mk));             // outside the image: real zero
                    }
                } else if (m < m_end) {
                    const int iy0 = pk_oh[i] * a.stride - a.pad, ix0 = pk_ow[i] * a.stride - a.pad;
                    const int8_t *base = a.X + (((size_t)pk_b[i] * a.H + iy0) * a.W + ix0) * a.C;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        // branch-free: lanes without a source read the tensor's first word and drop it
                        const int iy = iy0 + pk_r[d], ix = ix0 + pk_s[d];
                        const bool in = pk_r[d] >= 0 && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                        const int x = *reinterpret_cast<const int *>(in ? base + pk_off[d] : a.X);
                        v[d] = in ? x : pk_r[d] >= 0 ? fill : 0;
                    }
                }
                pk_ow[i] += MB;
                while (pk_ow[i] >= a.OW) { pk_ow[i] -= a.OW; pk_oh[i]++; }
                while (pk_oh[i] >= a.OH) { pk_oh[i] -= a.OH; pk_b[i]++; }
            } else if (m < m_end && c < a.C) {
                int ow, oh, b;                                    // (a division costs some 40 instructions, three a stage's worth of MFMAs)
                if (a.magic_ok) {
                    const unsigned t = hq_magic_div((unsigned)m, a.magic_OW), bb = hq_magic_div(t, a.magic_OH);
                    ow = (int)((unsigned)m - t * (unsigned)a.OW); oh = (int)(t - bb * (unsigned)a.OH); b = (int)bb;
                } else {
                    ow = m % a.OW; oh = (m / a.OW) % a.OH; b = m / (a.OW * a.OH);
                }
                const int iy = oh * a.stride - a.pad + tr, ix = ow * a.stride - a.pad + ts;
                if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) {
                    v = load16(a.X + (((size_t)b * a.H + iy) * a.W + ix) * a.C + c, a.C - c, a.x16);
                } else {
                    // real zero; bytes past the last channel stay 0 so they add nothing to xsum
                    const int nb = a.C - c;
                    v[0] = nb > 0 ? fill : 0; v[1] = nb > 4 ? fill : 0; v[2] = nb > 8 ? fill : 0; v[3] = nb > 12 ? fill : 0;
                }
            }
            xreg[i] = v;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < GLD; i++) {
            const int idx = tid + i * HQ_THREADS, row = idx / GCH, col = (idx % GCH) * 16;
            *reinterpret_cast<v4i *>(&Gs[buf][row * PG + col]) = greg[i];
        }
#pragma unroll
        for (int i = 0; i < XLD; i++) {
            const int idx = tid + i * HQ_THREADS, row = idx / XCH, col = (idx % XCH) * 16;
            *reinterpret_cast<v4i *>(&Xs[buf][row * PX + col]) = xreg[i];
        }
    };

    v16i acc[NT][KT];
#pragma unroll
    for (int i = 0; i < NT; i++)
#pragma unroll
        for (int j = 0; j < KT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0;
    int gs[NT], xs[KT];
#pragma unroll
    for (int i = 0; i < NT; i++) gs[i] = 0;
#pragma unroll
    for (int j = 0; j < KT; j++) xs[j] = 0;

    if (m_begin < m_end) {
        const int stages = (m_end - m_begin + MB - 1) / MB;
        load_stage(m_begin);
        store_stage(0);
        __syncthreads();
        for (int st = 0; st < stages; st++) {
            const int buf = st & 1;
            const bool more = st + 1 < stages;
            if (more) load_stage(m_begin + (st + 1) * MB);
#pragma unroll
            for (int ks = 0; ks < MB / 32; ks++) {
                v4i gf[NT], xf[KT];
#pragma unroll
                for (int i = 0; i < NT; i++)
                    gf[i] = read_frag_tr<PG>(&Gs[buf][ks * 32 * PG + wn * WTN + i * 32], lane);
#pragma unroll
                for (int j = 0; j < KT; j++)
                    xf[j] = read_frag_tr<PX>(&Xs[buf][ks * 32 * PX + wk * WTK + j * 32], lane);
#pragma unroll
                for (int i = 0; i < NT; i++)
#pragma unroll
                    for (int j = 0; j < KT; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gf[i], xf[j], acc[i][j], 0, 0, 0);
                if (do_gsum) {
#pragma unroll
                    for (int i = 0; i < NT; i++)
#pragma unroll
                        for (int d = 0; d < 4; d++) gs[i] = __builtin_amdgcn_sdot4(gf[i][d], 0x01010101, gs[i], false);
                }
                if (do_xsum) {
#pragma unroll
                    for (int j = 0; j < KT; j++)
#pragma unroll
                        for (int d = 0; d < 4; d++) xs[j] = __builtin_amdgcn_sdot4(xf[j][d], 0x01010101, xs[j], false);
                }
            }
            if (more) store_stage(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- merge the partial tile.  G fragments were the first MFMA operand: lane l holds
    // column c = l % 32 of the block and rows n = 8*(r/4) + 4*(l/32) + r%4.
    const size_t krow = (size_t)a.R * a.S * a.C;
#pragma unroll
    for (int i = 0; i < NT; i++)
#pragma unroll
        for (int j = 0; j < KT; j++) {
            int c = c0 + wk * WTK + j * 32 + (lane & 31);
            if (PACKED3) c = (c >> 5) < a.R && (c & 31) < a.S * 3 ? (c >> 5) * a.S * 3 + (c & 31) : kcols;   // tile column -> weight column
            if (c >= (PACKED ? kcols : a.C)) continue;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int n = n0 + wn * WTN + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (n >= a.N) continue;
                int32_t *dst = a.acc + (size_t)n * krow + (size_t)tap * a.C + c;
                if (a.direct) *dst = acc[i][j][r];
                else if (acc[i][j][r] != 0) atomicAdd(dst, acc[i][j][r]);
            }
        }
    if (do_gsum) {
#pragma unroll
        for (int i = 0; i < NT; i++) {
            int s = gs[i] + __shfl_xor(gs[i], 32);
            const int n = n0 + wn * WTN + i * 32 + (lane & 31);
            if (lane < 32 && n < a.N && s != 0) atomicAdd(a.gsum + n, s);
        }
    }
    if (do_xsum) {
#pragma unroll
        for (int j = 0; j < KT; j++) {
            int s = xs[j] + __shfl_xor(xs[j], 32);
            int c = c0 + wk * WTK + j * 32 + (lane & 31);
            if (PACKED3) c = (c >> 5) < a.R && (c & 31) < a.S * 3 ? (c >> 5) * a.S * 3 + (c & 31) : kcols;
            if (lane < 32 && c < (PACKED ? kcols : a.C) && s != 0) atomicAdd(a.xsum + (size_t)tap * a.C + c, s);
        }
    }
}

// ---------------------------------------------------------------------------------------
// 3x3, stride 1, pad 1, C % 64 == 0 and Cout % 64 == 0: the shape of most layers of the paper's
// networks (Table 5; ResNet-18 basic blocks).  One workgroup owns a 64 (Cout) x 64 (C) block of
// G_W for all nine taps (36 MFMA tiles, in registers for the whole launch) and walks a run of
// pixel bands.  A band (a few output rows of one image, or a few whole small images) is
// staged once: the dY rows as they lie in memory and the input rows with their one-pixel
// border; the nine taps are nine shifted views of that input patch, so an input byte is
// fetched once per band instead of once per tap.
// The reduction index of an MFMA k-step is the output pixel; the transposing LDS read takes
// a row address per lane, so each lane looks up the patch row of its pixels in a small
// table (pixel -> row of tap (0,0)) and adds the tap's offset.
// 512 threads: two groups of four wavefronts take alternate k-steps of a band (both groups
// accumulate the same 36 tiles and are added through LDS at the end); inside a group a
// wavefront owns one 32-channel block of C and taps 0..4 or 5..8 for both 32-blocks of Cout:
// 7 fragments feed 10 MFMAs.
// ---------------------------------------------------------------------------------------
// Weight gradient of a network's first layer (3 or 4 input channels, even stride, W a multiple of 4, at most
// 8 taps per filter row, at most 64 output channels in multiples of 16) with the input rows staged in LDS.
// A workgroup walks bands of whole output rows.  The input rows of a band are copied into LDS once, every
// pixel widened to 4 bytes, inside a frame of zero-point pixels; filter row r of output pixel (oy, ox) is then
// the 32 bytes at (oy * stride + r) * pitch + 4 * stride * ox: rows of an implicit [pixel][32 columns] matrix
// with a pitch of 4 * stride bytes, which the transposing LDS read takes as they lie (column 4 s + c of
// filter row r; the columns of the fourth byte and of taps past S are dropped at the end).  The gradient rows
// of the band are copied beside them.  Wavefront (wn, wk) owns output channels 32 wn .. 32 wn + 31 and filter
// rows 4 wk .. 4 wk + 3; sums stay in registers over all bands of the workgroup and leave with one atomic
// add per value.
struct WstemArgs {
    WgradArgs w;
    int rows_out, in_rows, LP;     // output rows per band, input rows it needs, LDS pitch of an input row
    int xrows;                     // input rows a buffer has room for: (rows_out - 1) * stride + 8
    int bands_per_image, nbands;
    int groups;                    // 16-byte groups of four pixels per input row: W / 4
    unsigned magic_groups, magic_OW;
    int gpitch, gchunks;           // LDS pitch of a gradient row, 16-byte chunks of a gradient row that are staged
    int kpad;                      // pixels of a full band rounded up to 32
};
constexpr int WS_XT = 3;           // staged groups of four pixels per thread and band
constexpr int WS_GT = 4;           // staged 16-byte gradient chunks per thread and band

template <int CH>
__global__ __launch_bounds__(HQ_THREADS, 2) void hq_wgrad_stem_kernel(const WstemArgs sa)
{
    const WgradArgs &a = sa.w;
    extern __shared__ __attribute__((aligned(16))) int8_t ws_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wn = wave >> 1, wk = wave & 1;
    const int zx = a.xq->zero_point;
    const int fill = (int)((unsigned)(zx & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const int xbytes = sa.xrows * sa.LP, gbytes = sa.kpad * sa.gpitch, buf_bytes = xbytes + gbytes;
    int8_t *zero_row = ws_lds + 2 * (size_t)buf_bytes;              // 64 bytes of 0: the source of pixels past a band
    const bool do_gsum = wk == 0 && zx != 0;                        // column sums of G (times z_x later)
    const bool do_xsum = wn == 0 && a.gq->zero_point != 0;          // column sums of the gathered input

    // the frame: the input part of both buffers starts as zero-point pixels; staging only writes the W image
    // columns of a row
    for (int b = 0; b < 2; b++)
        for (int q = tid; q < xbytes / 16; q += HQ_THREADS)
            *reinterpret_cast<v4i *>(ws_lds + (size_t)b * buf_bytes + (size_t)q * 16) = v4i{fill, fill, fill, fill};
    if (tid < 4) *reinterpret_cast<v4i *>(zero_row + tid * 16) = v4i{0, 0, 0, 0};

    int stx[WS_XT][CH];
    v4i stg[WS_GT];
    auto band_rows = [&](int band, int &b, int &oy0, int &nrows) {
        b = band / sa.bands_per_image;
        oy0 = (band - b * sa.bands_per_image) * sa.rows_out;
        nrows = min(sa.rows_out, a.OH - oy0);
    };
    // staging plan of this thread, the same for every band: its groups of four input pixels (input row of the
    // band, source offset from the band's first input row, LDS offset) and its 16-byte chunks of the gradient
    int x_row[WS_XT], x_src[WS_XT], x_dst[WS_XT];
#pragma unroll
    for (int k = 0; k < WS_XT; k++) {
        const int t = tid + k * HQ_THREADS;
        const int row = (int)hq_magic_div((unsigned)t, sa.magic_groups), g = t - row * sa.groups;
        x_row[k] = row < sa.in_rows ? row : -1;
        x_src[k] = (row * a.W + 4 * g) * CH;
        x_dst[k] = row * sa.LP + (a.pad + 4 * g) * 4;
    }
    int g_px[WS_GT], g_src[WS_GT], g_dst[WS_GT];
#pragma unroll
    for (int k = 0; k < WS_GT; k++) {
        const int t = tid + k * HQ_THREADS;
        const int px = t / sa.gchunks, cc = t - px * sa.gchunks;
        g_px[k] = px < sa.kpad && 16 * cc < a.N ? px : 0x7fffffff;        // never below a band's pixel count
        g_src[k] = px * a.N + 16 * cc;
        g_dst[k] = px < sa.kpad ? px * sa.gpitch + 16 * cc : -1;
    }
    auto stage_load = [&](int band) {
        int b, oy0, nrows;
        band_rows(band, b, oy0, nrows);
        const int iy0 = oy0 * a.stride - a.pad;
        const int8_t *xrow0 = a.X + ((ptrdiff_t)b * a.H + iy0) * a.W * CH;   // (may lie before the tensor: only rows inside are read)
#pragma unroll
        for (int k = 0; k < WS_XT; k++) {
            const int iy = iy0 + x_row[k];
            const bool ok = x_row[k] >= 0 && iy >= 0 && iy < a.H;
            const int8_t *src = ok ? xrow0 + x_src[k] : a.X;
#pragma unroll
            for (int c = 0; c < CH; c++) {
                const int x = reinterpret_cast<const int *>(src)[c];
                stx[k][c] = ok ? x : fill;
            }
        }
        const int npix = nrows * a.OW;
        const int8_t *g0 = a.G + ((size_t)b * a.OH + oy0) * a.OW * a.N;
#pragma unroll
        for (int k = 0; k < WS_GT; k++) {
            const bool ok = g_px[k] < npix;
            const v4i x = *reinterpret_cast<const v4i *>(ok ? g0 + g_src[k] : a.G);
            stg[k] = ok ? x : v4i{0, 0, 0, 0};
        }
    };
    auto stage_store = [&](int buf) {
        int8_t *xb = ws_lds + (size_t)buf * buf_bytes, *gb = xb + xbytes;
#pragma unroll
        for (int k = 0; k < WS_XT; k++) {
            if (x_row[k] < 0) continue;
            v4i v;
            if (CH == 4) {
                v = v4i{stx[k][0], stx[k][1], stx[k][2], stx[k][3]};
            } else {
                const unsigned w0 = (unsigned)stx[k][0], w1 = (unsigned)stx[k][1], w2 = (unsigned)stx[k][2];
                v[0] = (int)w0;
                v[1] = (int)__builtin_amdgcn_alignbyte(w1, w0, 3);
                v[2] = (int)__builtin_amdgcn_alignbyte(w2, w1, 2);
                v[3] = (int)(w2 >> 8);
            }
            *reinterpret_cast<v4i *>(xb + x_dst[k]) = v;
        }
#pragma unroll
        for (int k = 0; k < WS_GT; k++)
            if (g_dst[k] >= 0) *reinterpret_cast<v4i *>(gb + g_dst[k]) = stg[k];
    };

    v16i acc[4];
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[j][e] = 0;
    int gs = 0, xs[4] = {0, 0, 0, 0};

    const int per = (sa.nbands + gridDim.x - 1) / gridDim.x;
    const int band_begin = blockIdx.x * per, band_end = min(sa.nbands, band_begin + per);
    __syncthreads();
    if (band_begin < band_end) {
        stage_load(band_begin);
        stage_store(0);
    }
    __syncthreads();
    // transposing read: lane l hands in the address of 8 bytes (columns 16 * grp + 8 * (j & 1) ..) of pixel row
    // half * 16 + j / 2 (and of the row 8 further down) and receives column l % 32 of the 16 pixels of its half
    const int tj = lane & 15, tgrp = (lane >> 4) & 1, thalf = lane >> 5;
    const int tcol = 16 * tgrp + 8 * (tj & 1);
    typedef LDS_PTR(int8_t) lds_bytes;
    const lds_bytes lds0 = (lds_bytes)ws_lds;
    const unsigned zero_off = 2u * (unsigned)buf_bytes + (unsigned)tcol;
    for (int band = band_begin; band < band_end; band++) {
        const int buf = (band - band_begin) & 1;
        int b, oy0, nrows;
        band_rows(band, b, oy0, nrows);
        const int npix = nrows * a.OW, nks = (npix + 31) / 32;
        if (band + 1 < band_end) stage_load(band + 1);
        const unsigned xoff = (unsigned)buf * (unsigned)buf_bytes, goff = xoff + (unsigned)xbytes;
        // fragments of k-step ks: the gradient block and the wavefront's four filter rows (rows past R read rows
        // of the buffer that exist but hold anything: their sums are dropped at the end)
        auto load_frags = [&](int ks, v4i &gf, v4i (&xf)[4]) {
            const unsigned g0 = goff + (unsigned)((ks * 32 + thalf * 16 + (tj >> 1)) * sa.gpitch + wn * 32 + tcol);
            const tr_v2i glo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(lds0 + g0));
            const tr_v2i ghi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(lds0 + g0 + 8 * sa.gpitch));
            gf = v4i{glo[0], glo[1], ghi[0], ghi[1]};
            unsigned pa[2], pstep[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int px = ks * 32 + thalf * 16 + (tj >> 1) + 8 * h;
                const bool ok = px < npix;
                const unsigned q = ok ? (unsigned)px : 0u;
                const unsigned orow = hq_magic_div(q, sa.magic_OW), ox = q - orow * (unsigned)a.OW;
                pa[h] = ok ? xoff + (orow * (unsigned)a.stride + (unsigned)(wk * 4)) * (unsigned)sa.LP + 4u * (unsigned)a.stride * ox + (unsigned)tcol
                           : zero_off;
                pstep[h] = ok ? (unsigned)sa.LP : 0u;
            }
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const tr_v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(lds0 + pa[0] + j * pstep[0]));
                const tr_v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(lds0 + pa[1] + j * pstep[1]));
                xf[j] = v4i{lo[0], lo[1], hi[0], hi[1]};
            }
        };
        auto multiply = [&](const v4i &gf, const v4i (&xf)[4]) {
#pragma unroll
            for (int j = 0; j < 4; j++) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gf, xf[j], acc[j], 0, 0, 0);
            if (do_gsum) {
#pragma unroll
                for (int d = 0; d < 4; d++) gs = __builtin_amdgcn_sdot4(gf[d], 0x01010101, gs, false);
            }
            if (do_xsum) {
#pragma unroll
                for (int j = 0; j < 4; j++)
#pragma unroll
                    for (int d = 0; d < 4; d++) xs[j] = __builtin_amdgcn_sdot4(xf[j][d], 0x01010101, xs[j], false);
            }
        };
        // two fragment sets: the next k-step's reads are on their way while this one is multiplied
        v4i gfA, gfB, xfA[4], xfB[4];
        if (nks > 0) load_frags(0, gfA, xfA);
        for (int ks = 0; ks < nks; ks += 2) {
            if (ks + 1 < nks) load_frags(ks + 1, gfB, xfB);
            multiply(gfA, xfA);
            if (ks + 1 >= nks) break;
            if (ks + 2 < nks) load_frags(ks + 2, gfA, xfA);
            multiply(gfB, xfB);
        }
        if (band + 1 < band_end) stage_store(buf ^ 1);
        __syncthreads();
    }

    // ---- flush.  G fragments were the first MFMA operand: lane l holds column l % 32 of the filter row and
    // output channels 8 * (e / 4) + 4 * (l / 32) + e % 4 of the wavefront's block
    const size_t krow = (size_t)a.R * a.S * CH;
    const int col = lane & 31, tap = col >> 2, ch = col & 3;
    const bool col_ok = tap < a.S && ch < CH;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int r = wk * 4 + j;
        if (r >= a.R || !col_ok) continue;
        const size_t wc = ((size_t)r * a.S + tap) * CH + ch;
#pragma unroll
        for (int e = 0; e < 16; e++) {
            const int n = wn * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (n < a.N && acc[j][e] != 0) atomicAdd(a.acc + (size_t)n * krow + wc, acc[j][e]);
        }
        if (do_xsum) {
            const int s = xs[j] + __shfl_xor(xs[j], 32);
            if (lane < 32 && s != 0) atomicAdd(a.xsum + wc, s);
        }
    }
    if (do_gsum) {
        const int s = gs + __shfl_xor(gs, 32);
        const int n = wn * 32 + (lane & 31);
        if (lane < 32 && n < a.N && s != 0) atomicAdd(a.gsum + n, s);
    }
}

// ---------------------------------------------------------------------------------------
constexpr int WB_THREADS = 512;
constexpr int WB_P = 96;               // LDS pitch of a 64-channel pixel row (32 mod 64: transposing reads)
constexpr int WB_XLD = 3, WB_GLD = 2;  // 16-byte chunks a thread stages per band (input patch / dY rows)
constexpr int WB_SLOT_V4 = 2 * 5 * 4 * 256;   // 16-byte words of one workgroup's partial sums
constexpr int WB_SUMS = 64 + 9 * 64;          // column sums a group of a workgroup leaves: dY [64], input [9][64]

struct WbandArgs {
    const int8_t *X, *G;
    const hq_qparams *xq, *gq;
    int32_t *partial;              // [slot][WB_SLOT_V4] 16-byte words: this workgroup's 64 x 9 x 64 sums
    int32_t *sums;                 // [slot][2 groups][64 + 9 * 64]: column sums of dY and of the input taps
    int B, H, W, C, N;
    int rows, nimg;                // band: `rows` output rows of one image, or `nimg` whole images (rows == H)
    int bands_per_img;
    unsigned magic_bpi;            // ceil(2^32 / bands_per_img)
    int nstages, stages_per_block, splits;
    int cparts, nparts;            // C / 64, N / 64
    int npix, npix_pad;            // output pixels of a band, rounded up to a k-step
    int prows, PW;                 // patch rows (nimg * (rows + 2)) and patch row length (W + 2)
    int xchunks, gchunks;          // 16-byte chunks of a patch / of a band of dY
    unsigned buf_bytes;            // one LDS buffer: patch + dY band
};

__global__ __launch_bounds__(WB_THREADS) void hq_wgrad_band_kernel(const WbandArgs a)
{
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    unsigned *tbl = reinterpret_cast<unsigned *>(smem);                 // [npix_pad] patch byte offset of pixel k
    int8_t *bufs = smem + ((a.npix_pad * 4 + 15) & ~15);
    const unsigned xbytes = (unsigned)a.prows * a.PW * WB_P;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: branches on it are uniform
    const int grp = wave >> 2, cblk = wave & 1, th = (wave >> 1) & 1;
    const int t0 = th ? 5 : 0, nt = th ? 4 : 5;

    // workgroup -> (output block, run of bands); the blocks of one run sit on one XCD
    int part, split;
    {
        const int per = a.cparts * a.nparts, total = per * a.splits;
        const int full = (total / (8 * per)) * (8 * per);
        if ((int)blockIdx.x < full) {
            const int g8 = blockIdx.x / (8 * per), r = blockIdx.x % (8 * per);
            split = g8 * 8 + (r & 7); part = r >> 3;
        } else {
            const int r = blockIdx.x - full;
            split = full / per + r / per; part = r % per;
        }
    }
    const int cp = part % a.cparts, np = part / a.cparts;
    const int c0 = cp * 64, n0 = np * 64;
    const int s_begin = split * a.stages_per_block, s_end = min(a.nstages, s_begin + a.stages_per_block);
    const int zx = a.xq->zero_point;
    const int fillw = (int)((unsigned)(zx & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    // a column sum is only ever multiplied by the other operand's zero point (the finalize kernel's
    // correction terms): with that zero point at 0 it is not formed at all
    const bool do_gsum = cp == 0 && cblk == 0 && th == 0 && zx != 0;
    const bool do_xsum = np == 0 && a.gq->zero_point != 0;

    // ---- per-thread staging plan (the same for every band)
    int x_rel[WB_XLD], x_rowimg[WB_XLD];                 // source offset; patch row | image << 16
    bool x_on[WB_XLD], x_col[WB_XLD];
#pragma unroll
    for (int i = 0; i < WB_XLD; i++) {
        const int idx = tid + WB_THREADS * i, c16 = idx & 3, ppix = idx >> 2;
        const int prow = ppix / a.PW, pcol = ppix - prow * a.PW;
        x_on[i] = idx < a.xchunks;
        const int il = prow / (a.rows + 2), pr = prow - il * (a.rows + 2);
        x_rowimg[i] = pr | (il << 16);
        x_col[i] = pcol >= 1 && pcol <= a.W;
        x_rel[i] = ((il * a.H + pr - 1) * a.W + (pcol - 1)) * a.C + c16 * 16;
    }
    int g_rel[WB_GLD], g_il[WB_GLD];
    bool g_on[WB_GLD];
#pragma unroll
    for (int i = 0; i < WB_GLD; i++) {
        const int idx = tid + WB_THREADS * i, c16 = idx & 3, p = idx >> 2;
        g_on[i] = idx < a.gchunks;
        g_il[i] = p / (a.rows * a.W);
        g_rel[i] = p * a.N + c16 * 16;
    }
    v4i xreg[WB_XLD], greg[WB_GLD];
    auto load_stage = [&](int s) {
        int b0, y0;
        if (a.nimg == 1) { b0 = (int)hq_magic_div((unsigned)s, a.magic_bpi); y0 = (s - b0 * a.bands_per_img) * a.rows; }
        else { b0 = s * a.nimg; y0 = 0; }
        const size_t pix0 = ((size_t)b0 * a.H + y0) * a.W;
        const int8_t *xs = a.X + pix0 * a.C + c0;
        const int8_t *gs = a.G + pix0 * a.N + n0;
#pragma unroll
        for (int i = 0; i < WB_XLD; i++) {
            const bool img = b0 + (x_rowimg[i] >> 16) < a.B;        // images past the end of the batch count as zeros
            const bool inside = img && x_col[i] && (unsigned)(y0 + (x_rowimg[i] & 0xffff) - 1) < (unsigned)a.H;
            const int f = img ? fillw : 0;                          // border of a real image: real zero
            v4i v = {f, f, f, f};
            if (x_on[i] && inside) v = *reinterpret_cast<const v4i *>(xs + x_rel[i]);
            xreg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < WB_GLD; i++) {
            v4i v = {0, 0, 0, 0};
            if (g_on[i] && b0 + g_il[i] < a.B) v = *reinterpret_cast<const v4i *>(gs + g_rel[i]);
            greg[i] = v;
        }
    };
    auto store_stage = [&](int buf) {
        int8_t *xb = bufs + buf * a.buf_bytes, *gb = xb + xbytes;
#pragma unroll
        for (int i = 0; i < WB_XLD; i++)
            if (x_on[i]) {
                const int idx = tid + WB_THREADS * i;
                *reinterpret_cast<v4i *>(xb + (idx >> 2) * WB_P + (idx & 3) * 16) = xreg[i];
            }
#pragma unroll
        for (int i = 0; i < WB_GLD; i++)
            if (g_on[i]) {
                const int idx = tid + WB_THREADS * i;
                *reinterpret_cast<v4i *>(gb + (idx >> 2) * WB_P + (idx & 3) * 16) = greg[i];
            }
    };

    // ---- start-up: first band on its way, pixel table, zero rows behind the last pixel of a band
    if (s_begin < s_end) load_stage(s_begin);
    for (int k = tid; k < a.npix_pad; k += WB_THREADS) {
        unsigned off = 0;                                  // pixels past the band read patch row 0 (their dY is zero)
        if (k < a.npix) {
            const int il = k / (a.rows * a.W), rem = k - il * a.rows * a.W;
            const int oy = rem / a.W, ox = rem - oy * a.W;
            off = (unsigned)(((il * (a.rows + 2) + oy) * a.PW + ox) * WB_P);
        }
        tbl[k] = off;
    }
    for (int i = tid; i < (a.npix_pad - a.npix) * (WB_P / 4) * 2; i += WB_THREADS) {
        const int buf = i / ((a.npix_pad - a.npix) * (WB_P / 4)), w = i % ((a.npix_pad - a.npix) * (WB_P / 4));
        reinterpret_cast<int *>(bufs + buf * a.buf_bytes + xbytes + a.npix * WB_P)[w] = 0;
    }
    if (s_begin < s_end) store_stage(0);
    __syncthreads();

    v16i acc[2][5];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int u = 0; u < 5; u++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][u][r] = 0;
    int gsv[2] = {0, 0}, xsv[5] = {0, 0, 0, 0, 0};

    // lane's place in a fragment: rows klo and klo + 8 of the k-step, 8 bytes at column `fcol`
    const int j16 = lane & 15;
    const int klo = (lane >> 5) * 16 + (j16 >> 1);
    const int fcol = 16 * ((lane >> 4) & 1) + 8 * (j16 & 1);
    unsigned tapoff[5];
#pragma unroll
    for (int u = 0; u < 5; u++) {
        const int t = min(t0 + u, 8);
        tapoff[u] = (unsigned)(((t / 3) * a.PW + (t % 3)) * WB_P) + cblk * 32 + fcol;
    }
    const int nks = a.npix_pad / 32, ninv = a.npix_pad - a.npix;

    for (int s = s_begin; s < s_end; s++) {
        const int it = s - s_begin, buf = it & 1;
        const bool more = s + 1 < s_end;
        if (more) load_stage(s + 1);
        const int8_t *xb = bufs + buf * a.buf_bytes, *gb = xb + xbytes;
        for (int ks = (grp + it) & 1; ks < nks; ks += 2) {
            const int kb = ks * 32;
            const unsigned rlo = tbl[kb + klo], rhi = tbl[kb + klo + 8];
            v4i gf[2], xf[5];
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int8_t *p = gb + (kb + klo) * WB_P + i * 32 + fcol;
                const tr_v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(p));
                const tr_v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(p + 8 * WB_P));
                gf[i] = v4i{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int u = 0; u < 5; u++) {
                if (u < nt) {
                    const tr_v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(xb + rlo + tapoff[u]));
                    const tr_v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(tr_v2i))(xb + rhi + tapoff[u]));
                    xf[u] = v4i{lo[0], lo[1], hi[0], hi[1]};
                }
            }
            // the column sums ride behind the MFMAs of their own fragment (four dot products per tap, in the
            // shadow of the matrix cores); issued after all ten MFMAs they would hold up the next k-step
#pragma unroll
            for (int u = 0; u < 5; u++) {
                if (u < nt) {
#pragma unroll
                    for (int i = 0; i < 2; i++)
                        acc[i][u] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gf[i], xf[u], acc[i][u], 0, 0, 0);
                    if (do_xsum) {
#pragma unroll
                        for (int d = 0; d < 4; d++) xsv[u] = __builtin_amdgcn_sdot4(xf[u][d], 0x01010101, xsv[u], false);
                    }
                    if (do_gsum && u < 2) {
#pragma unroll
                        for (int d = 0; d < 4; d++) gsv[u] = __builtin_amdgcn_sdot4(gf[u][d], 0x01010101, gsv[u], false);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the band's last k-step read patch row 0 for its `ninv` pixels past the band: take that back
        // (in the group that took that k-step)
        if (do_xsum && ninv > 0 && ((nks - 1 - grp - it) & 1) == 0 && lane < 32) {
#pragma unroll
            for (int u = 0; u < 5; u++)
                if (u < nt) xsv[u] -= ninv * (int)xb[tapoff[u] - fcol + (lane & 31)];
        }
        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- add the two groups through LDS, one 32-block of Cout per round (the group that
    // receives alternates), and store this workgroup's partial sums with plain 16-byte stores:
    // partial[slot][i][u][r / 4][thread][r % 4].  The finalize kernel adds the slots; merging
    // with atomics instead would queue every workgroup of the launch on the same lines.
    int *xch = reinterpret_cast<int *>(smem);
    const int t256 = tid & 255;
    v4i *pout = reinterpret_cast<v4i *>(a.partial) + (size_t)(split * (a.cparts * a.nparts) + part) * WB_SLOT_V4;
#pragma unroll
    for (int i = 0; i < 2; i++) {
        if (grp != i) {
#pragma unroll
            for (int u = 0; u < 5; u++)
#pragma unroll
                for (int r = 0; r < 16; r++) xch[(u * 16 + r) * 256 + t256] = acc[i][u][r];
        }
        __syncthreads();
        if (grp == i) {
#pragma unroll
            for (int u = 0; u < 5; u++) {
                if (u < nt) {
#pragma unroll
                    for (int rq = 0; rq < 4; rq++) {
                        v4i v;
#pragma unroll
                        for (int e = 0; e < 4; e++) v[e] = acc[i][u][4 * rq + e] + xch[(u * 16 + 4 * rq + e) * 256 + t256];
                        pout[((i * 5 + u) * 4 + rq) * 256 + t256] = v;
                    }
                }
            }
        }
        __syncthreads();
    }
    // column sums: plain stores as well, one record per workgroup and group
    int *sp = a.sums + ((size_t)(split * (a.cparts * a.nparts) + part) * 2 + grp) * WB_SUMS;
    if (do_gsum) {
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int sm = gsv[i] + __shfl_xor(gsv[i], 32);
            if (lane < 32) sp[i * 32 + lane] = sm;
        }
    }
    if (do_xsum) {
#pragma unroll
        for (int u = 0; u < 5; u++) {
            if (u < nt) {
                const int sm = xsv[u] + __shfl_xor(xsv[u], 32);
                if (lane < 32) sp[64 + (t0 + u) * 64 + cblk * 32 + lane] = sm;
            }
        }
    }
}

__global__ void zero_kernel(int32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Removes the zero points (32-bit wrap-around arithmetic is exact as long as the true
// result fits 32 bits) and applies the one FP32 scale.
__global__ void wgrad_finalize_kernel(const int32_t *acc, const int32_t *gsum, const int32_t *xsum,
                                      const hq_qparams *xq, const hq_qparams *gq, unsigned M, int N, int K,
                                      int gsum_per_k, float *dW, int32_t *dW_acc, const HqRideAlong ride)
{
    if (hq_ride_along(ride)) return;
    const unsigned zx = (unsigned)xq->zero_point, zg = (unsigned)gq->zero_point;
    const float s = __fmul_rn(xq->scale, gq->scale);
    const size_t total = (size_t)N * K;
    const unsigned nblocks = ride.n ? (unsigned)ride.first : gridDim.x;       // workgroups doing this kernel's own work
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)nblocks * blockDim.x) {
        const int n = (int)(i / K), k = (int)(i % K);
        const unsigned g = (unsigned)gsum[gsum_per_k ? k % gsum_per_k : n];
        unsigned c = (unsigned)acc[i] - zx * g - zg * (unsigned)xsum[k] + M * zx * zg;
        if (dW_acc) dW_acc[i] = (int)c;
        dW[i] = __fmul_rn(s, (float)(int)c);
    }
}


// Band kernel's finalize: adds the workgroups' partial sums (64 threads along C, TY taking every
// TY-th slot), removes the zero points and scales.  One thread owns 4 consecutive output
// channels of one (tap, c): the 16 bytes a lane of the band kernel stored.
template <int TY>
__global__ __launch_bounds__(64 * TY) void wband_finalize_kernel(const int32_t *partial, const int32_t *sums,
                                                              const hq_qparams *xq, const hq_qparams *gq, unsigned M,
                                                              int N, int C, int splits, float *dW, int32_t *dW_acc,
                                                              const HqRideAlong ride)
{
    if (hq_ride_along(ride)) return;
    __shared__ v4i sh[TY][64];
    __shared__ int shx[TY][64], shg[TY][4];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int cparts = C / 64, parts = cparts * (N / 64);
    const size_t o = (size_t)blockIdx.x * 64 + tx;                 // (n / 4, tap, c), c fastest
    const int c = (int)(o % C), tap = (int)((o / C) % 9), n0 = (int)(o / ((size_t)9 * C)) * 4;
    const int cp = c / 64, cblk = (c >> 5) & 1, np = n0 / 64, i = (n0 >> 5) & 1, rq = (n0 >> 3) & 3, lh = (n0 >> 2) & 1;
    const int th = tap >= 5, u = tap - 5 * th;
    const int t256 = (th * 2 + cblk) * 64 + lh * 32 + (c & 31);
    const v4i *src = reinterpret_cast<const v4i *>(partial) + (size_t)(np * cparts + cp) * WB_SLOT_V4 +
                     ((i * 5 + u) * 4 + rq) * 256 + t256;
    const int *xsrc = sums + (size_t)cp * 2 * WB_SUMS + 64 + tap * 64 + (c & 63);            // workgroups with np == 0
    const int *gsrc = sums + (size_t)(np * cparts) * 2 * WB_SUMS + (n0 & 63) + (tx & 3);    // workgroups with cp == 0
    v4i sum = {0, 0, 0, 0};
    int xs = 0, gs = 0;
    // a column sum is only ever multiplied by the other operand's zero point: with that at 0 it is neither formed
    // by the band kernel nor read here (uniform branches)
    const bool need_xs = gq->zero_point != 0, need_gs = xq->zero_point != 0;
    for (int s = ty; s < splits; s += TY) {
        sum += src[(size_t)s * parts * WB_SLOT_V4];
        const size_t so = (size_t)s * parts * 2 * WB_SUMS;
        if (need_xs) xs += xsrc[so] + xsrc[so + WB_SUMS];
        if (need_gs && tx < 4) gs += gsrc[so] + gsrc[so + WB_SUMS];
    }
    sh[ty][tx] = sum; shx[ty][tx] = xs;
    if (tx < 4) shg[ty][tx] = gs;
    __syncthreads();
    if (ty != 0) return;
    int g4[4] = {0, 0, 0, 0};
#pragma unroll
    for (int y = 1; y < TY; y++) { sum += sh[y][tx]; xs += shx[y][tx]; }
#pragma unroll
    for (int y = 0; y < TY; y++)
#pragma unroll
        for (int e = 0; e < 4; e++) g4[e] += shg[y][e];
    const unsigned zx = (unsigned)xq->zero_point, zg = (unsigned)gq->zero_point;
    const float sc = __fmul_rn(xq->scale, gq->scale);
    const size_t K = (size_t)9 * C, k = (size_t)tap * C + c;
    const unsigned xterm = zg * (unsigned)xs, both = M * zx * zg;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const unsigned v = (unsigned)sum[e] - zx * (unsigned)g4[e] - xterm + both;
        const size_t idx = (size_t)(n0 + e) * K + k;
        if (dW_acc) dW_acc[idx] = (int)v;
        dW[idx] = __fmul_rn(sc, (float)(int)v);
    }
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// Geometry of the band kernel for one layer (host, pure); covered == false: the tile kernel takes it.
struct WbandPlan {
    bool covered;
    int rows, nimg, nstages, stages_per_block, splits, parts;
    int npix, npix_pad, prows;
    size_t lds, buf_bytes;
};

WbandPlan wband_plan(const hq_problem *p)
{
    WbandPlan pl = {};
    if (p->kind != HQ_CONV2D || p->R != 3 || p->S != 3 || p->stride != 1 || p->pad != 1) return pl;
    if (p->C % 64 != 0 || p->Cout % 64 != 0) return pl;
    const int H = p->H, W = p->W;
    // candidates: `rows` output rows of one image (rows | H), or `nimg` whole images; a band holds at
    // most 256 pixels and what 512 threads stage in WB_XLD / WB_GLD chunks each.  Prefer the band
    // that wastes the fewest k-steps (the two groups take ceil(nks / 2) k-steps per band).
    int best_rows = 0, best_nimg = 0;
    double best_eff = 0.0;
    auto consider = [&](int rows, int nimg) {
        const int npix = nimg * rows * W, prows = nimg * (rows + 2);
        if (npix > 256 || npix * 4 > WB_GLD * WB_THREADS || prows * (W + 2) * 4 > WB_XLD * WB_THREADS) return;
        const int nks = (npix + 31) / 32;
        const double eff = (double)npix / (64.0 * ((nks + 1) / 2));
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && npix > best_nimg * best_rows * W)) {
            best_eff = eff; best_rows = rows; best_nimg = nimg;
        }
    };
    for (int rows = 1; rows <= H; rows++) if (H % rows == 0) consider(rows, 1);
    for (int nimg = 2; nimg * H * W <= 256; nimg++) consider(H, nimg);
    if (best_rows == 0) return pl;
    pl.rows = best_rows; pl.nimg = best_nimg;
    pl.nstages = best_nimg == 1 ? p->B * (H / best_rows) : (p->B + best_nimg - 1) / best_nimg;
    pl.parts = (p->C / 64) * (p->Cout / 64);
    pl.npix = best_nimg * best_rows * W; pl.npix_pad = (pl.npix + 31) & ~31;
    pl.prows = best_nimg * (best_rows + 2);
    pl.buf_bytes = (size_t)pl.prows * (W + 2) * WB_P + (size_t)pl.npix_pad * WB_P;
    pl.lds = (size_t)((pl.npix_pad * 4 + 15) & ~15) + 2 * pl.buf_bytes;
    const size_t reduce_bytes = 5 * 16 * 256 * 4;           // the two groups meet in LDS at the end
    if (pl.lds < reduce_bytes) pl.lds = reduce_bytes;
    if (pl.lds > 160 * 1024) return pl;
    int splits = pl.parts >= 256 ? 1 : (256 + pl.parts - 1) / pl.parts;     // one workgroup per compute unit
    if (splits > pl.nstages) splits = pl.nstages;
    pl.stages_per_block = (pl.nstages + splits - 1) / splits;
    pl.splits = (pl.nstages + pl.stages_per_block - 1) / pl.stages_per_block;
    pl.covered = true;
    return pl;
}

size_t wband_partial_bytes(const WbandPlan &pl) { return pl.covered ? (size_t)pl.parts * pl.splits * WB_SLOT_V4 * 16 : 0; }
size_t wband_sums_bytes(const WbandPlan &pl) { return pl.covered ? (size_t)pl.parts * pl.splits * 2 * WB_SUMS * 4 : 0; }

bool launch_wgrad_band(const hq_problem *p, const WbandPlan &pl, const WgradArgs &w, int32_t *partial, int32_t *sums,
                       hipStream_t stream)
{
    WbandArgs a;
    a.X = w.X; a.G = w.G; a.xq = w.xq; a.gq = w.gq; a.partial = partial; a.sums = sums;
    a.B = p->B; a.H = p->H; a.W = p->W; a.C = p->C; a.N = p->Cout;
    a.rows = pl.rows; a.nimg = pl.nimg;
    a.bands_per_img = p->H / pl.rows;
    a.magic_bpi = hq_magic32((unsigned)a.bands_per_img);
    a.nstages = pl.nstages; a.stages_per_block = pl.stages_per_block; a.splits = pl.splits;
    a.cparts = p->C / 64; a.nparts = p->Cout / 64;
    a.npix = pl.npix; a.npix_pad = pl.npix_pad;
    a.prows = pl.prows; a.PW = p->W + 2;
    a.xchunks = a.prows * a.PW * 4; a.gchunks = a.npix * 4;
    a.buf_bytes = (unsigned)pl.buf_bytes;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(hq_wgrad_band_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return false;
        configured = true;
    }
    hipLaunchKernelGGL(hq_wgrad_band_kernel, dim3((unsigned)(pl.parts * pl.splits)), dim3(WB_THREADS), pl.lds, stream, a);
    return true;
}

} // namespace

// Workspace: [Cout][K] integer sums, [Cout] and [K] column sums, then the band kernel's partial sums.
size_t hq_wgrad_workspace_bytes(const hq_problem *p)
{
    const size_t K = (size_t)p->R * p->S * p->C;
    if (p->kind == HQ_DEPTHWISE) return align16(4 * K) + align16(4 * (size_t)p->C) + align16(4 * K);
    return align16(4 * (size_t)p->Cout * K) + align16(4 * (size_t)p->Cout) + align16(4 * K) +
           wband_partial_bytes(wband_plan(p)) + wband_sums_bytes(wband_plan(p));
}

int hq_launch_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                    const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, hipStream_t stream,
                    const HqRideAlong *ride)
{
    HqRideAlong ra = {nullptr, nullptr, 0, 0};
    if (ride) ra = *ride;
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    const size_t K = (size_t)p->R * p->S * p->C;
    WgradArgs a;
    a.X = X; a.G = dY; a.xq = xq; a.gq = gq;
    char *w = static_cast<char *>(ws);
    a.acc = reinterpret_cast<int32_t *>(w);
    const size_t acc_bytes = align16(4 * (size_t)p->Cout * K);
    a.gsum = reinterpret_cast<int32_t *>(w + acc_bytes);
    a.xsum = reinterpret_cast<int32_t *>(w + acc_bytes + align16(4 * (size_t)p->Cout));
    const size_t sums_bytes = acc_bytes + align16(4 * (size_t)p->Cout) + align16(4 * K);
    a.M = p->B * OH * OW; a.N = p->Cout; a.C = p->C;
    a.R = p->R; a.S = p->S; a.H = p->H; a.W = p->W; a.OH = OH; a.OW = OW; a.stride = p->stride; a.pad = p->pad;
    a.g16 = (a.N % 16) == 0; a.x16 = (a.C % 16) == 0;
    a.magic_ok = (unsigned long long)a.M * (unsigned long long)(OW > OH ? OW : OH) < (1ull << 32);   // hq_magic_div's range
    a.magic_OW = a.magic_ok ? hq_magic32((unsigned)OW) : 0u;
    a.magic_OH = a.magic_ok ? hq_magic32((unsigned)OH) : 0u;

    const WbandPlan pl = wband_plan(p);
    if (pl.covered) {
        // every workgroup stores its sums to a slot of its own: nothing to zero, no atomics
        int32_t *partial = reinterpret_cast<int32_t *>(w + sums_bytes);
        int32_t *sums = reinterpret_cast<int32_t *>(w + sums_bytes + wband_partial_bytes(pl));
        if (!launch_wgrad_band(p, pl, a, partial, sums, stream)) return HQ_E_HIP;
        const size_t quads = (size_t)a.N / 4 * K;              // multiple of 64 (C % 64 == 0)
        ra.first = (int)(quads / 64);
        const dim3 fgrid((unsigned)(quads / 64) + (unsigned)ra.n);
        if (pl.splits >= 48)
            hipLaunchKernelGGL(wband_finalize_kernel<16>, fgrid, dim3(1024), 0, stream, partial, sums, xq, gq,
                               (unsigned)a.M, a.N, a.C, pl.splits, dW, dW_acc, ra);
        else if (pl.splits >= 12)
            hipLaunchKernelGGL(wband_finalize_kernel<4>, fgrid, dim3(256), 0, stream, partial, sums, xq, gq,
                               (unsigned)a.M, a.N, a.C, pl.splits, dW, dW_acc, ra);
        else
            hipLaunchKernelGGL(wband_finalize_kernel<1>, fgrid, dim3(64), 0, stream, partial, sums, xq, gq,
                               (unsigned)a.M, a.N, a.C, pl.splits, dW, dW_acc, ra);
        return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
    }

    // first layers on even strides: input rows staged in LDS (hq_wgrad_stem_kernel)
    if ((a.C == 3 || a.C == 4) && p->stride % 2 == 0 && p->W % 4 == 0 && p->S <= 8 && p->R <= 8 && a.N <= 64 &&
        a.N % 16 == 0 && (reinterpret_cast<uintptr_t>(X) & 3) == 0 && (reinterpret_cast<uintptr_t>(dY) & 15) == 0) {
        WstemArgs sa;
        sa.w = a;
        sa.w.direct = 0;
        const int lp_reads = 4 * (OW - 1) * p->stride + 32, lp_image = 4 * (p->W + p->pad);
        sa.LP = ((lp_reads > lp_image ? lp_reads : lp_image) + 15) & ~15;
        sa.groups = p->W / 4;
        sa.magic_groups = hq_magic32((unsigned)sa.groups);
        sa.magic_OW = hq_magic32((unsigned)OW);
        const int nb32 = (a.N + 31) / 32;
        sa.gpitch = nb32 * 32 + 32;
        sa.gchunks = nb32 * 2;
        int rows = 0;
        for (int r = 1; r <= OH; r++) {
            const int in_rows = (r - 1) * p->stride + p->R, kpad = (r * OW + 31) / 32 * 32;
            if ((size_t)((r - 1) * p->stride + 8) * sa.LP + (size_t)kpad * sa.gpitch > 39 * 1024 || in_rows * sa.groups > WS_XT * HQ_THREADS ||
                kpad * sa.gchunks > WS_GT * HQ_THREADS)
                break;
            rows = r;
        }
        if (rows >= 1 && (unsigned long long)p->B * OH * OW < (1ull << 31)) {
            sa.rows_out = rows;
            sa.in_rows = (rows - 1) * p->stride + p->R;
            sa.xrows = (rows - 1) * p->stride + 8;
            sa.kpad = (rows * OW + 31) / 32 * 32;
            sa.bands_per_image = (OH + rows - 1) / rows;
            sa.nbands = p->B * sa.bands_per_image;
            const size_t lds = 2 * ((size_t)sa.xrows * sa.LP + (size_t)sa.kpad * sa.gpitch) + 64;
            static bool configured = false;
            if (!configured) {
                if (hipFuncSetAttribute(reinterpret_cast<const void *>(hq_wgrad_stem_kernel<3>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024) != hipSuccess ||
                    hipFuncSetAttribute(reinterpret_cast<const void *>(hq_wgrad_stem_kernel<4>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024) != hipSuccess)
                    return HQ_E_HIP;
                configured = true;
            }
            const size_t zwords = sums_bytes / 4;
            hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((zwords + 255) / 256 > 1024 ? 1024 : (zwords + 255) / 256)),
                               dim3(256), 0, stream, a.acc, zwords);
            const int sblocks = sa.nbands < 512 ? sa.nbands : 512;
            if (a.C == 3) hipLaunchKernelGGL(hq_wgrad_stem_kernel<3>, dim3(sblocks), dim3(HQ_THREADS), lds, stream, sa);
            else          hipLaunchKernelGGL(hq_wgrad_stem_kernel<4>, dim3(sblocks), dim3(HQ_THREADS), lds, stream, sa);
            const size_t total = (size_t)a.N * K;
            unsigned fb = (unsigned)((total + 255) / 256 > 2048 ? 2048 : (total + 255) / 256);
            ra.first = (int)fb;
            hipLaunchKernelGGL(wgrad_finalize_kernel, dim3(fb + (unsigned)ra.n), dim3(256), 0, stream, a.acc, a.gsum, a.xsum,
                               xq, gq, (unsigned)a.M, a.N, (int)K, 0, dW, dW_acc, ra);
            return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
        }
    }

    const bool big = a.N > 64 && a.C > 64, packed = a.C < 16;
    const int TN = big ? 128 : 64, TK = packed ? 256 : big ? 128 : 64;
    a.ctiles = (a.C + TK - 1) / TK;
    // (3-channel inputs: 32 tile columns per filter row)
    const int xt = a.C == 3 ? (p->R * 32 + TK - 1) / TK : packed ? (int)((K + TK - 1) / TK) : p->R * p->S * a.ctiles;
    const int yt = (a.N + TN - 1) / TN;
    const int stages_total = (a.M + MB - 1) / MB;
    // Workgroups to aim at.  Small tiles need many resident workgroups to hide their stage latency;
    // 128x128 tiles carry 64 KB of atomics each, and those queue on the same lines when every split
    // finishes at once, so they get longer runs of pixels and fewer splits.
    // (first layers: three resident workgroups per compute unit; more splits only add atomics: 256 against 283 us
    // on the 7x7 stride-2 stem at batch 256)
    const int target = packed ? 768 : !big ? 2048 : p->R * p->S == 1 ? 256 : 512;
    int splits = (target + xt * yt - 1) / (xt * yt);
    if (splits > stages_total) splits = stages_total;
    // (a run shorter than about ten stages is mostly start-up and atomics: a 1x1 stride-2 layer 64 -> 128 at
    // 28x28 outputs, batch 256, takes 26 us with runs of 12 stages against 42 us with runs of 3)
    if (!big && !packed && splits > stages_total / 10) {
        const int fill = (512 + xt * yt - 1) / (xt * yt);          // but keep two workgroups per compute unit
        splits = stages_total / 10 > fill ? stages_total / 10 : splits < fill ? splits : fill;
    }
    if (splits < 1) splits = 1;
    const int stages_per = (stages_total + splits - 1) / splits;
    a.m_per_split = stages_per * MB;
    splits = (stages_total + stages_per - 1) / stages_per;
    a.xt = xt; a.yt = yt; a.splits = splits;
    // one split: the tiles partition [N][K], so the sums are stored, not added, and only the column sums start at zero
    a.direct = splits == 1 && !packed;
    int32_t *zero_from = a.direct ? a.gsum : a.acc;
    const size_t ws_words = (a.direct ? sums_bytes - acc_bytes : sums_bytes) / 4;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((ws_words + 255) / 256 > 1024 ? 1024 : (ws_words + 255) / 256)),
                       dim3(256), 0, stream, zero_from, ws_words);
    dim3 grid((unsigned)(xt * yt * splits));
    if (a.C == 3) hipLaunchKernelGGL((hq_wgrad_kernel<64, 256, true, true>), grid, dim3(HQ_THREADS), 0, stream, a);
    else if (packed) hipLaunchKernelGGL((hq_wgrad_kernel<64, 256, true>), grid, dim3(HQ_THREADS), 0, stream, a);
    else if (big) hipLaunchKernelGGL((hq_wgrad_kernel<128, 128, false>), grid, dim3(HQ_THREADS), 0, stream, a);
    else          hipLaunchKernelGGL((hq_wgrad_kernel<64, 64, false>), grid, dim3(HQ_THREADS), 0, stream, a);

    const size_t total = (size_t)a.N * K;
    unsigned fb = (unsigned)((total + 255) / 256 > 2048 ? 2048 : (total + 255) / 256);
    ra.first = (int)fb;
    hipLaunchKernelGGL(wgrad_finalize_kernel, dim3(fb + (unsigned)ra.n), dim3(256), 0, stream, a.acc, a.gsum, a.xsum, xq, gq,
                       (unsigned)a.M, a.N, (int)K, 0, dW, dW_acc, ra);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}
