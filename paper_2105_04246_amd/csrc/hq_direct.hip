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
    int blocks = (a.tiles + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    const bool fused = out32 == nullptr;
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
