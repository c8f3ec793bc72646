// Forward GEMM of a network's first layer (3 or 4 input channels, e.g. the 7x7 stride-2 stem on RGB
// images, or on images padded to 4 channels) on int8 MFMA with the fused in-hindsight epilogue (paper Sec. 3.1,
// Sec. 3.2 static quantization, Sec. 4 steps 1 and 2).
//
// In NHWC the S taps of one filter row are S * C contiguous bytes of the input, and with
// S * C <= 32 they are one MFMA k-step: the reduction is laid out as R k-steps of 32 bytes (filter
// row r = k-step r; bytes past S * C meet zero weights).  A lane's 16 bytes of an input fragment
// are then 16 contiguous bytes of memory, so the fragments are loaded straight from global memory
// into registers (4-byte loads, each with its own bounds test; neighbouring pixels overlap in
// cache), with no staging through LDS and no gather arithmetic beyond one row pointer per k-step.
// The weight fragments of all R k-steps stay in registers for the whole launch.  The output is
// large compared with the input (64 channels out of 4), so the kernel is bound by the epilogue's
// vector-ALU work and by the HBM write of the codes.
// With 3 channels a pixel is 3 bytes, so a lane's 4-byte words start at any byte address and a word
// can hold bytes of two taps: words are loaded unaligned and the bytes whose tap lies outside the
// image (or past the filter row) are replaced under a per-word byte mask.  The 16 bytes themselves come
// from aligned loads of the words that hold them and a byte-wise funnel shift.
#include "hq_device.h"
#include "hq_internal.h"
#include <type_traits>

namespace {

constexpr int DR_MAXR = 7;         // filter rows held in registers
constexpr int DR_MI = 1;           // 32-pixel blocks per tile of a wavefront

struct DirectArgs {
    const int8_t *A, *Bw;
    const int32_t *bsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int M, N, C, R, S, H, W, Ho, Wo, stride, pad, Bn;
    unsigned magic_Wo, magic_Ho;   // ceil(2^32 / d)
    int tiles;                     // tiles of 32 * DR_MI pixels
};

__device__ inline int dr_sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

// NT: 32-channel blocks of the output (N <= 32 * NT).  CH: input channels, 4 (a tap is one aligned word) or 3.
template <int NT, bool FUSED, int CH>
__global__ __launch_bounds__(HQ_THREADS, 2) void hq_direct_kernel(const DirectArgs a)
{
    __shared__ int red[4 * (HQ_THREADS / 64)];
    __shared__ __attribute__((aligned(16))) int bzs[32 * NT];       // z_a * bsum[n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5;
    const int za = a.aq->zero_point;
    const int fill = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const int rowbytes = a.S * a.C;                     // valid bytes of a k-step
    if (tid < 32 * NT) bzs[tid] = tid < a.N ? za * a.bsum[tid] : 0;

    // weight fragments: lane holds output channel j*32 + sigma(lane % 32) (so that the accumulators
    // of a lane are 16 consecutive channels), bytes 16*half .. +15 of filter row r
    v4i wf[DR_MAXR][NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        const int n = j * 32 + dr_sigma32(lane & 31);
#pragma unroll
        for (int r = 0; r < DR_MAXR; r++) {
            v4i v = {0, 0, 0, 0};
            if (r < a.R && n < a.N) {
                const int8_t *w = a.Bw + ((size_t)n * a.R + r) * rowbytes + 16 * half;
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    if (CH == 4) {
                        if (16 * half + 4 * d < rowbytes) v[d] = *reinterpret_cast<const int *>(w + 4 * d);
                    } else {
                        const unsigned mk = hq_bytemask(0, rowbytes - (16 * half + 4 * d));     // bytes of this filter row
                        const v4i x = hq_load16_any(w, a.Bw, a.Bw + (size_t)a.N * a.R * rowbytes);
                        v[d] = (int)((unsigned)x[d] & mk);
                    }
                }
            }
            wf[r][j] = v;
        }
    }
    __syncthreads();

    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;

    // input fragments of one tile: [filter row][32-pixel block]
    auto load_frags = [&](int tile, v4i (&af)[DR_MAXR][DR_MI]) {
#pragma unroll
        for (int i = 0; i < DR_MI; i++) {
            const int m = tile * (32 * DR_MI) + i * 32 + (lane & 31);
            const bool ok = tile < a.tiles && m < a.M;
            const unsigned mm = ok ? (unsigned)m : 0u;
            const unsigned t = hq_magic_div(mm, a.magic_Wo), ox = mm - t * a.Wo;         // t = b * Ho + oy
            const unsigned b = hq_magic_div(t, a.magic_Ho), oy = t - b * a.Ho;
            const int iy0 = (int)oy * a.stride - a.pad;
            if (CH == 4) {
                const int ix0 = (int)ox * a.stride - a.pad + 4 * half;                       // C == 4: tap = word
                const int8_t *p0 = a.A + ((size_t)b * a.H * a.W + ix0) * a.C;
                bool wok[4];
#pragma unroll
                for (int d = 0; d < 4; d++) wok[d] = ok && 4 * half + d < a.S && ix0 + d >= 0 && ix0 + d < a.W;
#pragma unroll
                for (int r = 0; r < DR_MAXR; r++) {
                    // every lane loads (lanes without a source read the tensor's first word instead and
                    // drop it): no branch per word, and the loads of a tile issue back to back
                    v4i v;
                    const int iy = iy0 + r;
                    const bool rok = r < a.R && iy >= 0 && iy < a.H;
                    const int8_t *p = p0 + (ptrdiff_t)iy * a.W * a.C;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        const bool k = rok && wok[d];
                        const int x = *reinterpret_cast<const int *>(k ? p + 4 * d : a.A);
                        v[d] = k ? x : fill;
                    }
                    af[r][i] = v;
                }
            } else {
                // byte k of the k-step is channel k % 3 of tap k / 3: the taps inside the image and the filter
                // row are the bytes k0 <= k < k1, the same for every filter row of this pixel
                const int ixb = (int)ox * a.stride - a.pad;
                const int k0 = CH * max(0, -ixb), k1 = CH * min(a.S, a.W - ixb);
                unsigned mk[4];
#pragma unroll
                for (int d = 0; d < 4; d++) mk[d] = ok ? hq_bytemask(k0 - (16 * half + 4 * d), k1 - (16 * half + 4 * d)) : 0u;
                const int8_t *p0 = a.A + ((ptrdiff_t)b * a.H * a.W + ixb) * CH + 16 * half;
                const int8_t *aend = a.A + (size_t)a.Bn * a.H * a.W * CH;
#pragma unroll
                for (int r = 0; r < DR_MAXR; r++) {
                    const int iy = iy0 + r;
                    const bool rok = ok && r < a.R && iy >= 0 && iy < a.H;
                    const v4i x = hq_load16_any(rok ? p0 + (ptrdiff_t)iy * a.W * CH : a.A, a.A, aend);
                    v4i v;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        const unsigned m = rok ? mk[d] : 0u;
                        v[d] = (int)(((unsigned)x[d] & m) | ((unsigned)fill & ~m));
                    }
                    af[r][i] = v;
                }
            }
        }
    };
    auto process = [&](int tile, const v4i (&af)[DR_MAXR][DR_MI]) {
        v16i acc[DR_MI][NT];
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const v4i bz = *reinterpret_cast<const v4i *>(bzs + j * 32 + 16 * half + 4 * g);
#pragma unroll
                for (int i = 0; i < DR_MI; i++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[i][j][4 * g + e] = -bz[e];
            }
#pragma unroll
        for (int r = 0; r < DR_MAXR; r++) {
            if (r < a.R) {
#pragma unroll
                for (int i = 0; i < DR_MI; i++)
#pragma unroll
                    for (int j = 0; j < NT; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[r][j], af[r][i], acc[i][j], 0, 0, 0);
            }
        }
        auto epilogue = [&](auto full) {
            constexpr bool FULL = decltype(full)::value;
#pragma unroll
            for (int i = 0; i < DR_MI; i++) {
                const int m = tile * (32 * DR_MI) + i * 32 + (lane & 31);
                if (m >= a.M) continue;
#pragma unroll
                for (int j = 0; j < NT; j++) {
                    const int nb = j * 32 + 16 * half;
                    if (nb >= a.N) continue;                           // N % 16 == 0: a group is all in or all out
                    int c[16];
#pragma unroll
                    for (int e = 0; e < 16; e++) c[e] = acc[i][j][e];
                    const size_t o = (size_t)m * a.N + nb;
                    if (FUSED) {
                        int w[4];
                        hq_requant_group<16, FULL>(c, ep, mn, mx, nlo, nhi, w);
                        const v4i v = {w[0], w[1], w[2], w[3]};
                        *reinterpret_cast<v4i *>(a.out8 + o) = v;
                    } else {
                        hq_minmax_group<16>(c, mn, mx);
#pragma unroll
                        for (int g = 0; g < 4; g++) {
                            const v4i v = {c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                            *reinterpret_cast<v4i *>(a.out32 + o + 4 * g) = v;
                        }
                    }
                }
            }
        };
        if (ep.full_grid) epilogue(std::true_type()); else epilogue(std::false_type());
    };

    // two register sets: the next tile's fragments are on their way while this tile is multiplied
    // and requantized
    const int wave_global = blockIdx.x * (HQ_THREADS / 64) + wave, nwaves = gridDim.x * (HQ_THREADS / 64);
    v4i afA[DR_MAXR][DR_MI], afB[DR_MAXR][DR_MI];
    int tile = wave_global;
    if (tile < a.tiles) load_frags(tile, afA);
    while (tile < a.tiles) {
        load_frags(tile + nwaves, afB);
        process(tile, afA);
        tile += nwaves;
        if (tile >= a.tiles) break;
        load_frags(tile + nwaves, afA);
        process(tile, afB);
        tile += nwaves;
    }
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.N);
        if (FUSED) *a.outq = a.range->qp;
    }
}


// ---------------------------------------------------------------------------------------------------------
// The same layer with the input rows staged in LDS (even stride, W * C a multiple of 4): a workgroup walks
// bands of whole output rows; the input rows a band needs are copied once into LDS with every pixel widened
// to 4 bytes (3-channel pixels: three funnel shifts per four pixels; the fourth byte meets a zero weight)
// inside a frame of zero-point pixels, so a lane's 16 bytes of an input fragment are two aligned 8-byte
// LDS reads at (input row) * pitch + 4 * stride * ox, with no bounds logic and no byte masks.  The k-step of
// filter row r is then tap s at bytes 4 s .. 4 s + 3 (weights of the fourth byte and of taps past S are 0).
// The next band's rows are on their way (global -> registers) while this band is multiplied.
struct StemArgs {
    DirectArgs d;
    int rows_out;                  // output rows per band
    int in_rows;                   // (rows_out - 1) * stride + R
    int LP;                        // LDS row pitch in bytes (multiple of 16)
    int bands_per_image, nbands;
    int groups;                    // 16-byte groups of four pixels per input row: W / 4
    unsigned magic_groups;
};

constexpr int ST_TASKS = 5;        // staged 4-pixel groups per thread and band (host checks the fit)

template <int NT, bool FUSED, int CH>
__global__ __launch_bounds__(HQ_THREADS, 2) void hq_stem_kernel(const StemArgs sa)
{
    const DirectArgs &a = sa.d;
    extern __shared__ __attribute__((aligned(16))) int8_t stem_lds[];
    __shared__ int red[4 * (HQ_THREADS / 64)];
    __shared__ __attribute__((aligned(16))) int bzs[32 * NT];       // -z_a * bsum[n]: what the accumulators start from
    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int za = a.aq->zero_point;
    const int fill = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const int buf_bytes = sa.in_rows * sa.LP;
    if (tid < 32 * NT) bzs[tid] = tid < a.N ? -(za * a.bsum[tid]) : 0;
    // the frame: every word of both buffers starts as zero-point pixels; staging only ever writes the W image
    // columns of a row, so the columns left and right of the image keep this value
    for (int q = tid; q < 2 * buf_bytes / 16; q += HQ_THREADS)
        *reinterpret_cast<v4i *>(stem_lds + (size_t)q * 16) = v4i{fill, fill, fill, fill};

    // weight fragments in the widened layout: byte 4 s + c of k-step r is W[n][r][s][c] (c < CH, s < S), else 0
    v4i wf[DR_MAXR][NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        const int n = j * 32 + dr_sigma32(lane & 31);
#pragma unroll
        for (int r = 0; r < DR_MAXR; r++) {
            v4i v = {0, 0, 0, 0};
            if (r < a.R && n < a.N) {
                const int8_t *w = a.Bw + ((size_t)n * a.R + r) * a.S * CH;
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    const int s = 4 * half + d;
                    unsigned x = 0;
                    if (s < a.S) {
#pragma unroll
                        for (int c = 0; c < CH; c++) x |= (unsigned)(uint8_t)w[s * CH + c] << (8 * c);
                    }
                    v[d] = (int)x;
                }
            }
            wf[r][j] = v;
        }
    }

    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;

    // ---- staging: task = (input row of the band, group of four pixels); words held between load and store
    int stw[ST_TASKS][CH];
    auto band_rows = [&](int band, int &b, int &oy0, int &nrows) {
        b = band / sa.bands_per_image;
        oy0 = (band - b * sa.bands_per_image) * sa.rows_out;
        nrows = min(sa.rows_out, a.Ho - oy0);
    };
    auto stage_load = [&](int band) {
        int b, oy0, nrows;
        band_rows(band, b, oy0, nrows);
        const int iy0 = oy0 * a.stride - a.pad;
#pragma unroll
        for (int k = 0; k < ST_TASKS; k++) {
            const int t = tid + k * HQ_THREADS;
            const int row = (int)hq_magic_div((unsigned)t, sa.magic_groups), g = t - row * sa.groups;
            const int iy = iy0 + row;
            const bool ok = band < sa.nbands && row < sa.in_rows && iy >= 0 && iy < a.H;
            const int8_t *src = a.A + (ok ? (((size_t)b * a.H + iy) * a.W + 4 * g) * CH : 0);
#pragma unroll
            for (int c = 0; c < CH; c++) {
                const int x = reinterpret_cast<const int *>(src)[c];
                stw[k][c] = ok ? x : fill;
            }
        }
    };
    auto stage_store = [&](int buf) {
#pragma unroll
        for (int k = 0; k < ST_TASKS; k++) {
            const int t = tid + k * HQ_THREADS;
            const int row = (int)hq_magic_div((unsigned)t, sa.magic_groups), g = t - row * sa.groups;
            if (row >= sa.in_rows) continue;
            v4i v;
            if (CH == 4) {
                v = v4i{stw[k][0], stw[k][1], stw[k][2], stw[k][3]};
            } else {
                const unsigned w0 = (unsigned)stw[k][0], w1 = (unsigned)stw[k][1], w2 = (unsigned)stw[k][2];
                v[0] = (int)w0;                                         // p0: c0 c1 c2 (+ a byte of p1)
                v[1] = (int)__builtin_amdgcn_alignbyte(w1, w0, 3);      // p1
                v[2] = (int)__builtin_amdgcn_alignbyte(w2, w1, 2);      // p2
                v[3] = (int)(w2 >> 8);                                  // p3
            }
            *reinterpret_cast<v4i *>(stem_lds + (size_t)buf * buf_bytes + (size_t)row * sa.LP + (size_t)(a.pad + 4 * g) * 4) = v;
        }
    };

    // ---- fragments of one 32-pixel block of the band in buffer `buf`
    auto load_frags = [&](int buf, int blk, int npix, v4i (&af)[DR_MAXR][DR_MI]) {
        const int px = min(blk * 32 + (lane & 31), npix - 1);
        const int orow = (int)hq_magic_div((unsigned)px, a.magic_Wo), ox = px - orow * a.Wo;
        const int8_t *base = stem_lds + (size_t)buf * buf_bytes + (size_t)(orow * a.stride) * sa.LP + 4 * a.stride * ox + 16 * half;
#pragma unroll
        for (int r = 0; r < DR_MAXR; r++) {
            if (r < a.R) {
                const int2 lo = *reinterpret_cast<const int2 *>(base + (size_t)r * sa.LP);
                const int2 hi = *reinterpret_cast<const int2 *>(base + (size_t)r * sa.LP + 8);
                af[r][0] = v4i{lo.x, lo.y, hi.x, hi.y};
            }
        }
    };
    auto process = [&](size_t m0, int blk, int npix, const v4i (&af)[DR_MAXR][DR_MI]) {
        v16i acc[NT];
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const v4i bz = *reinterpret_cast<const v4i *>(bzs + j * 32 + 16 * half + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; e++) acc[j][4 * g + e] = bz[e];
            }
#pragma unroll
        for (int r = 0; r < DR_MAXR; r++) {
            if (r < a.R) {
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[r][j], af[r][0], acc[j], 0, 0, 0);
            }
        }
        auto epilogue = [&](auto full) {
            constexpr bool FULL = decltype(full)::value;
            const int px = blk * 32 + (lane & 31);
            if (px >= npix) return;
            const size_t m = m0 + px;
#pragma unroll
            for (int j = 0; j < NT; j++) {
                const int nb = j * 32 + 16 * half;
                if (nb >= a.N) continue;                           // N % 16 == 0: a group is all in or all out
                int c[16];
#pragma unroll
                for (int e = 0; e < 16; e++) c[e] = acc[j][e];
                const size_t o = m * a.N + nb;
                if (FUSED) {
                    int w[4];
                    hq_requant_group<16, FULL>(c, ep, mn, mx, nlo, nhi, w);
                    const v4i v = {w[0], w[1], w[2], w[3]};
                    *reinterpret_cast<v4i *>(a.out8 + o) = v;
                } else {
                    hq_minmax_group<16>(c, mn, mx);
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const v4i v = {c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                        *reinterpret_cast<v4i *>(a.out32 + o + 4 * g) = v;
                    }
                }
            }
        };
        if (ep.full_grid) epilogue(std::true_type()); else epilogue(std::false_type());
    };

    // ---- bands of this workgroup: a contiguous run
    const int per = (sa.nbands + gridDim.x - 1) / gridDim.x;
    const int band_begin = blockIdx.x * per, band_end = min(sa.nbands, band_begin + per);
    __syncthreads();                                       // frame and bzs written
    if (band_begin < band_end) {
        stage_load(band_begin);
        stage_store(0);
    }
    __syncthreads();
    for (int band = band_begin; band < band_end; band++) {
        const int buf = (band - band_begin) & 1;
        int b, oy0, nrows;
        band_rows(band, b, oy0, nrows);
        const int npix = nrows * a.Wo, nblk = (npix + 31) / 32;
        const size_t m0 = ((size_t)b * a.Ho + oy0) * a.Wo;
        if (band + 1 < band_end) stage_load(band + 1);
        v4i afA[DR_MAXR][DR_MI], afB[DR_MAXR][DR_MI];
        int blk = wave;
        if (blk < nblk) load_frags(buf, blk, npix, afA);
        while (blk < nblk) {
            if (blk + 4 < nblk) load_frags(buf, blk + 4, npix, afB);
            process(m0, blk, npix, afA);
            blk += 4;
            if (blk >= nblk) break;
            if (blk + 4 < nblk) load_frags(buf, blk + 4, npix, afA);
            process(m0, blk, npix, afB);
            blk += 4;
        }
        // the other buffer was last read in the previous band, behind whose closing barrier every wavefront is
        if (band + 1 < band_end) stage_store(buf ^ 1);
        __syncthreads();
    }
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.N);
        if (FUSED) *a.outq = a.range->qp;
    }
}

} // namespace

// Forward layers with 3 or 4 input channels, a filter row of at most 32 bytes, at most DR_MAXR filter
// rows and 16..64 output channels in multiples of 16; HQ_E_BADSHAPE means "not covered".
int hq_try_launch_direct(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                         const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                         int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream)
{
    if (dgrad || p->kind != HQ_CONV2D || (p->C != 4 && p->C != 3) || p->S * p->C > 32 || p->R > DR_MAXR) return HQ_E_BADSHAPE;
    if (p->Cout > 64 || p->Cout % 16 != 0) return HQ_E_BADSHAPE;
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    DirectArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.M = p->B * OH * OW; a.N = p->Cout; a.C = p->C; a.R = p->R; a.S = p->S; a.H = p->H; a.W = p->W;
    a.Ho = OH; a.Wo = OW; a.stride = p->stride; a.pad = p->pad; a.Bn = p->B;
    if ((unsigned long long)a.M * (unsigned long long)(OW > OH ? OW : OH) >= (1ull << 32)) return HQ_E_BADSHAPE;   // hq_magic_div's range
    a.magic_Wo = hq_magic32((unsigned)OW);
    a.magic_Ho = hq_magic32((unsigned)OH);
    a.tiles = (a.M + 32 * DR_MI - 1) / (32 * DR_MI);
    const bool fused = out32 == nullptr;
    // staged form: even stride (8-byte aligned fragment reads), rows that start on a word, 16-byte groups of
    // four pixels, at most 8 taps per filter row (a tap takes 4 bytes of the 32-byte k-step); the band is the largest run of output rows whose input rows fit two buffers of 31 KiB and
    // whose staging fits ST_TASKS groups per thread
    if (p->stride % 2 == 0 && p->W % 4 == 0 && p->S <= 8 && (reinterpret_cast<uintptr_t>(A) & 3) == 0) {
        StemArgs sa;
        sa.d = a;
        sa.LP = ((4 * (OW - 1) * p->stride + 32 > 4 * (p->W + p->pad) ? 4 * (OW - 1) * p->stride + 32 : 4 * (p->W + p->pad)) + 15) & ~15;
        sa.groups = p->W / 4;
        sa.magic_groups = hq_magic32((unsigned)sa.groups);
        int rows = 0;
        for (int r = 1; r <= OH && r <= 64; r++) {
            const int in_rows = (r - 1) * p->stride + p->R;
            if ((size_t)in_rows * sa.LP > 31 * 1024 || in_rows * sa.groups > ST_TASKS * HQ_THREADS) break;
            rows = r;
        }
        if (rows >= 1) {
            // prefer a band height that divides the image and fills whole 128-pixel rounds of the four wavefronts
            int best = rows;
            for (int r = rows; r >= 1 && r * 2 > rows; r--)
                if (OH % r == 0 && (r * OW) % 128 == 0) { best = r; break; }
            sa.rows_out = best;
            sa.in_rows = (best - 1) * p->stride + p->R;
            sa.bands_per_image = (OH + best - 1) / best;
            sa.nbands = p->B * sa.bands_per_image;
            const size_t lds = 2 * (size_t)sa.in_rows * sa.LP;
            int sblocks = sa.nbands < 512 ? sa.nbands : 512;
            auto slaunch = [&](auto kern) {
                hipLaunchKernelGGL(kern, dim3(sblocks), dim3(HQ_THREADS), lds, stream, sa);
            };
            if (p->C == 4) {
                if (a.N > 32) { if (fused) slaunch(hq_stem_kernel<2, true, 4>); else slaunch(hq_stem_kernel<2, false, 4>); }
                else          { if (fused) slaunch(hq_stem_kernel<1, true, 4>); else slaunch(hq_stem_kernel<1, false, 4>); }
            } else {
                if (a.N > 32) { if (fused) slaunch(hq_stem_kernel<2, true, 3>); else slaunch(hq_stem_kernel<2, false, 3>); }
                else          { if (fused) slaunch(hq_stem_kernel<1, true, 3>); else slaunch(hq_stem_kernel<1, false, 3>); }
            }
            return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
        }
    }
    int blocks = (a.tiles + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    auto launch = [&](auto kern) { hipLaunchKernelGGL(kern, dim3(blocks), dim3(HQ_THREADS), 0, stream, a); };
    if (p->C == 4) {
        if (a.N > 32) { if (fused) launch(hq_direct_kernel<2, true, 4>); else launch(hq_direct_kernel<2, false, 4>); }
        else          { if (fused) launch(hq_direct_kernel<1, true, 4>); else launch(hq_direct_kernel<1, false, 4>); }
    } else {
        if (a.N > 32) { if (fused) launch(hq_direct_kernel<2, true, 3>); else launch(hq_direct_kernel<2, false, 3>); }
        else          { if (fused) launch(hq_direct_kernel<1, true, 3>); else launch(hq_direct_kernel<1, false, 3>); }
    }
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}
