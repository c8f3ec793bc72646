// Weights-resident implicit-GEMM convolution for gfx950: the fast path of hq_gemm_fwd /
// hq_gemm_dgrad (and of pass 1 of the dynamic baseline) for layers whose quantized weights fit
// in LDS next to an input patch (paper Sec. 3.1 forward / backward linear op; Sec. 3.2 and Sec. 4
// for what the epilogue does).
//
// Mapping to the machine
//   * One workgroup (4 wavefronts) owns a band of output rows of one image and walks it in
//     tiles of 256 consecutive output pixels.  The layer's weights are copied to LDS once per
//     workgroup; two workgroups share a CU, so while one loads its next patch the other one
//     keeps the matrix cores busy.
//   * Per tile, the input rows the tile touches (with the zero-point code in the padding ring)
//     are staged in LDS once, as they lie in memory.  im2col never exists: each lane forms
//     the address of "its" pixel under tap (r,s) when it reads the MFMA fragment, so an input
//     byte crosses L2->LDS once per tile instead of once per tap.  The next tile's rows are
//     prefetched into registers while the current tile is multiplied.
//   * v_mfma_i32_32x32x32_i8 with the weights as first operand: a lane then holds one output
//     pixel and, because the weight rows are stored in LDS in permuted order, 16 CONSECUTIVE
//     output channels, so the epilogue stores 16 codes (or 16 accumulators) per lane at once.
//   * Epilogue per accumulator: subtract z_a * bsum[n]; fold into per-lane min / max; count
//     clipped values with two integer compares against thresholds found once per kernel by
//     bisection on the exact fp32 requantization formula (it is monotone), the counts
//     accumulating in scalar registers through wavefront ballots; requantize with one fp32
//     multiply, round-half-even, clamp, and pack.
#include "hq_device.h"
#include "hq_internal.h"

namespace {

struct BandArgs {
    const int8_t *A, *Bw;
    const int32_t *bsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int N, npad;                   // output channels, rounded up to the column tile
    int Hs, Ws, Ho, Wo;            // source image, output image
    int stride, pad, flip;         // effective padding; flip = weight taps mirrored (dgrad)
    int PW, PRmax;                 // patch width (pixels), most patch rows any tile needs
    int rows_per_band, bands_per_image;
    unsigned magic_Wo, magic_row;  // ceil(2^32 / Wo), ceil(2^32 / (PW * C/16))
    unsigned long long count;      // outputs of the whole tensor
};

constexpr int BM = 256;            // output pixels per tile: 4 wavefronts x 2 MFMA row blocks

__device__ inline int sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

template <int C> __device__ inline int wswz(int i)
{
    return (C % 128 == 0) ? (i & 7) : (C % 64 == 0) ? ((i >> 1) & 3) : ((i >> 2) & 1);
}

// Largest accumulator value that does not clip high / smallest that does not clip low.
__device__ inline int clip_threshold(float mult, float bound, bool high)
{
    auto inside = [&](long long c) {
        float r = rintf(__fmul_rn((float)(int)c, mult));
        return high ? r <= bound : r >= bound;
    };
    long long good = 0, bad = high ? (long long)INT_MAX + 1 : (long long)INT_MIN - 1;   // c = 0 never clips
    if (inside(high ? INT_MAX : INT_MIN)) return high ? INT_MAX : INT_MIN;
    while ((high ? bad - good : good - bad) > 1) {
        long long mid = good + (bad - good) / 2;
        if (inside(mid)) good = mid; else bad = mid;
    }
    return (int)good;
}

template <int C, int KSZ, int NT, int NPF, bool FUSED>
__global__ __launch_bounds__(HQ_THREADS, 2) void hq_band_kernel(const BandArgs a)
{
    constexpr int NCH = C / 16, KS = C / 32, PP = C + 16, BN = 32 * NT, TAPS = KSZ * KSZ;
    constexpr int WROW = TAPS * C;                        // bytes per weight row in LDS
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t *Wl = smem;                                     // [npad][TAPS][C], chunks swizzled
    int *bz = reinterpret_cast<int *>(smem + (size_t)a.npad * WROW);     // [npad]  z_a * bsum[n]
    int8_t *Pl = reinterpret_cast<int8_t *>(bz + a.npad);  // [PRmax * PW][PP]
    int *red = reinterpret_cast<int *>(Pl + (size_t)a.PRmax * a.PW * PP);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int za = a.aq->zero_point;
    const int fillw = (za & 0xff) * 0x01010101;
    const v4i fill = {fillw, fillw, fillw, fillw};

    // ---- weights and zero-point terms: once per workgroup
    for (int idx = tid; idx < a.npad * TAPS * NCH; idx += HQ_THREADS) {
        const int cq = idx % NCH, t = (idx / NCH) % TAPS, row = idx / (NCH * TAPS);
        const int i = row & 31, n = (row & ~31) + sigma32(i);
        const int tsrc = a.flip ? TAPS - 1 - t : t;
        v4i v = {0, 0, 0, 0};
        if (n < a.N) v = *reinterpret_cast<const v4i *>(a.Bw + ((size_t)n * TAPS + tsrc) * C + cq * 16);
        *reinterpret_cast<v4i *>(Wl + row * WROW + t * C + 16 * (cq ^ wswz<C>(i))) = v;
    }
    for (int n = tid; n < a.npad; n += HQ_THREADS) bz[n] = n < a.N ? za * a.bsum[n] : 0;

    // ---- requantization constants
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqRequant rq = {1.0f, 0.0f, 0.0f, 0};
    int c_lo = INT_MIN, c_hi = INT_MAX;
    if (FUSED) {
        rq = hq_make_requant(acc_scale, a.range->qp, a.range->qlo, a.range->qhi);
        c_hi = clip_threshold(rq.mult, rq.fhi, true);
        c_lo = clip_threshold(rq.mult, rq.flo, false);
    }
    const float zoff = (float)(rq.z + 128);

    // ---- this workgroup's band
    const int img = blockIdx.x / a.bands_per_image, band = blockIdx.x % a.bands_per_image;
    const int row0 = band * a.rows_per_band, row1 = min(a.Ho, row0 + a.rows_per_band);
    const int p0 = row0 * a.Wo, p1 = row1 * a.Wo;
    const int8_t *Aimg = a.A + (size_t)img * a.Hs * a.Ws * C;
    const size_t out_img = (size_t)img * a.Ho * a.Wo;
    const int rowchunks = a.PW * NCH;

    v4i pf[NPF];
    auto prefetch = [&](int ps) {
        const int oy0 = ps / a.Wo, oy1 = (min(ps + BM, p1) - 1) / a.Wo;
        const int total = ((oy1 - oy0) * a.stride + KSZ) * rowchunks;
        const int iy_base = oy0 * a.stride - a.pad;
#pragma unroll
        for (int k = 0; k < NPF; k++) {
            const int idx = tid + HQ_THREADS * k;
            v4i v = fill;
            if (idx < total) {
                const int vr = (int)__umulhi((unsigned)idx, a.magic_row), rem = idx - vr * rowchunks;
                const int iy = iy_base + vr, ix = rem / NCH - a.pad, q = rem % NCH;
                if (iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws)
                    v = *reinterpret_cast<const v4i *>(Aimg + ((size_t)iy * a.Ws + ix) * C + q * 16);
            }
            pf[k] = v;
        }
    };
    auto stash = [&]() {
        const int cap = a.PRmax * rowchunks;
#pragma unroll
        for (int k = 0; k < NPF; k++) {
            const int idx = tid + HQ_THREADS * k;
            if (idx < cap) *reinterpret_cast<v4i *>(Pl + (idx / NCH) * PP + (idx % NCH) * 16) = pf[k];
        }
    };

    // per-lane weight fragment addresses (row i = lane % 32 of each 32-row block)
    int wbase[NT][KS];
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            wbase[j][ks] = (j * 32 + (lane & 31)) * WROW + 16 * ((ks * 2 + (lane >> 5)) ^ wswz<C>(lane & 31));

    int mn = INT_MAX, mx = INT_MIN;
    unsigned s_lo = 0, s_hi = 0;                           // wavefront-uniform clip counts

    prefetch(p0);
    for (int ps = p0; ps < p1; ps += BM) {
        __syncthreads();                                   // previous patch no longer read
        stash();
        __syncthreads();
        if (ps + BM < p1) prefetch(ps + BM);
        if (ps + wave * 64 >= p1) continue;                // this wavefront has no pixel in the tile

        const int oy0 = ps / a.Wo;
        int abase[2], pix[2];
        bool ok[2];
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int p = ps + wave * 64 + i * 32 + (lane & 31);
            ok[i] = p < p1;
            pix[i] = ok[i] ? p : ps;
            const int oy = (int)__umulhi((unsigned)pix[i], a.magic_Wo), ox = pix[i] - oy * a.Wo;
            abase[i] = (((oy - oy0) * a.stride) * a.PW + ox * a.stride) * PP + (lane >> 5) * 16;
        }

        for (int nc = 0; nc < a.npad / BN; nc++) {
            v16i acc[2][NT];
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < NT; j++)
#pragma unroll
                    for (int r = 0; r < 16; r++) acc[i][j][r] = 0;
            const int8_t *Wc = Wl + nc * BN * WROW;
#pragma unroll 1
            for (int r = 0; r < KSZ; r++)
#pragma unroll 1
                for (int s = 0; s < KSZ; s++) {
                    const int toff = (r * a.PW + s) * PP;
#pragma unroll
                    for (int ks = 0; ks < KS; ks++) {
                        v4i wf[NT], af[2];
#pragma unroll
                        for (int j = 0; j < NT; j++)
                            wf[j] = *reinterpret_cast<const v4i *>(Wc + wbase[j][ks] + (r * KSZ + s) * C);
#pragma unroll
                        for (int i = 0; i < 2; i++)
                            af[i] = *reinterpret_cast<const v4i *>(Pl + abase[i] + toff + ks * 32);
#pragma unroll
                        for (int i = 0; i < 2; i++)
#pragma unroll
                            for (int j = 0; j < NT; j++)
                                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], acc[i][j], 0, 0, 0);
                    }
                }

            // ---- epilogue: lane = one pixel, 16 consecutive channels per (row block, column block)
#pragma unroll
            for (int i = 0; i < 2; i++) {
                if (!ok[i]) continue;
                const size_t m = out_img + pix[i];
#pragma unroll
                for (int j = 0; j < NT; j++) {
                    const int nb = nc * BN + j * 32 + 16 * (lane >> 5);
                    if (nb >= a.N) continue;
                    v4i packed;
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const v4i bzv = *reinterpret_cast<const v4i *>(bz + nb + 4 * g);
                        int c[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            c[e] = acc[i][j][4 * g + e] - bzv[e];
                            mn = min(mn, c[e]); mx = max(mx, c[e]);
                        }
                        if (FUSED) {
                            unsigned w = 0;
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                s_hi += (unsigned)__popcll(__ballot(c[e] > c_hi));
                                s_lo += (unsigned)__popcll(__ballot(c[e] < c_lo));
                                float f = rintf(__fmul_rn((float)c[e], rq.mult));
                                f = __builtin_amdgcn_fmed3f(f, rq.flo, rq.fhi) + zoff;
                                w = __builtin_amdgcn_cvt_pk_u8_f32(f, e, w);
                            }
                            packed[g] = (int)(w ^ 0x80808080u);
                        } else {
                            const v4i v = {c[0], c[1], c[2], c[3]};
                            *reinterpret_cast<v4i *>(a.out32 + m * a.N + nb + 4 * g) = v;
                        }
                    }
                    if (FUSED) *reinterpret_cast<v4i *>(a.out8 + m * a.N + nb) = packed;
                }
            }
        }
    }

    __syncthreads();
    hq_block_stats_commit(mn, mx, lane == 0 ? s_lo : 0u, lane == 0 ? s_hi : 0u, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, a.count);
        if (FUSED) *a.outq = a.range->qp;
    }
}

unsigned magic32(unsigned d) { return (unsigned)(((1ull << 32) + d - 1) / d); }

template <int C, int KSZ, int NT, int NPF>
int launch_band(const BandArgs &a, int blocks, size_t lds, hipStream_t s)
{
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(hq_band_kernel<C, KSZ, NT, NPF, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(hq_band_kernel<C, KSZ, NT, NPF, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024) != hipSuccess)
            return HQ_E_HIP;
        configured = true;
    }
    if (a.out32 == nullptr)
        hipLaunchKernelGGL((hq_band_kernel<C, KSZ, NT, NPF, true>), dim3(blocks), dim3(HQ_THREADS), lds, s, a);
    else
        hipLaunchKernelGGL((hq_band_kernel<C, KSZ, NT, NPF, false>), dim3(blocks), dim3(HQ_THREADS), lds, s, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

} // namespace

// Returns HQ_OK after launching, HQ_E_BADSHAPE if this path does not cover the problem (the
// caller then uses the general gather kernel), HQ_E_HIP on a launch error.
int hq_try_launch_band(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                       const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                       int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream)
{
    if (p->kind != HQ_CONV2D || p->R != p->S) return HQ_E_BADSHAPE;
    if (dgrad && p->stride != 1) return HQ_E_BADSHAPE;
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    BandArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    int C;
    if (!dgrad) {
        C = p->C; a.N = p->Cout; a.Hs = p->H; a.Ws = p->W; a.Ho = OH; a.Wo = OW;
        a.stride = p->stride; a.pad = p->pad; a.flip = 0;
    } else {
        C = p->Cout; a.N = p->C; a.Hs = OH; a.Ws = OW; a.Ho = p->H; a.Wo = p->W;
        a.stride = 1; a.pad = p->R - 1 - p->pad; a.flip = 1;
    }
    const int KSZ = p->R;
    int NT, NPF;
    if (C == 64 && KSZ == 3) { NT = 2; NPF = 8; }
    else if (C == 32 && KSZ == 1) { NT = 2; NPF = 4; }
    else if (C == 192 && KSZ == 1) { NT = 1; NPF = 16; }
    else return HQ_E_BADSHAPE;
    if ((a.N % 16) != 0 || a.Ho * a.Wo >= 65536) return HQ_E_BADSHAPE;
    const int BN = 32 * NT;
    a.npad = (a.N + BN - 1) / BN * BN;
    a.PW = (a.Wo - 1) * a.stride + KSZ;

    // bands: at least two workgroups per CU when the batch allows it
    int bpi = (512 + p->B - 1) / p->B;
    if (bpi > a.Ho) bpi = a.Ho;
    if (bpi < 1) bpi = 1;
    a.rows_per_band = (a.Ho + bpi - 1) / bpi;
    a.bands_per_image = (a.Ho + a.rows_per_band - 1) / a.rows_per_band;
    // most patch rows any tile needs
    int prmax = 0;
    for (int band = 0; band < a.bands_per_image; band++) {
        const int r0 = band * a.rows_per_band, r1 = (r0 + a.rows_per_band < a.Ho) ? r0 + a.rows_per_band : a.Ho;
        for (int ps = r0 * a.Wo; ps < r1 * a.Wo; ps += BM) {
            const int last = (ps + BM < r1 * a.Wo ? ps + BM : r1 * a.Wo) - 1;
            const int rows = (last / a.Wo - ps / a.Wo) * a.stride + KSZ;
            if (rows > prmax) prmax = rows;
        }
    }
    a.PRmax = prmax;
    const int rowchunks = a.PW * (C / 16);
    if ((long)prmax * rowchunks > (long)NPF * HQ_THREADS) return HQ_E_BADSHAPE;
    if ((long)prmax * rowchunks >= 65536 || rowchunks >= 65536) return HQ_E_BADSHAPE;
    const size_t lds = (size_t)a.npad * KSZ * KSZ * C + (size_t)a.npad * 4 + (size_t)prmax * a.PW * (C + 16) + 64;
    if (lds > 80 * 1024) return HQ_E_BADSHAPE;
    a.magic_Wo = magic32((unsigned)a.Wo);
    a.magic_row = magic32((unsigned)rowchunks);
    a.count = (unsigned long long)p->B * a.Ho * a.Wo * a.N;
    const int blocks = p->B * a.bands_per_image;
    if (C == 64) return launch_band<64, 3, 2, 8>(a, blocks, lds, stream);
    if (C == 32) return launch_band<32, 1, 2, 4>(a, blocks, lds, stream);
    return launch_band<192, 1, 1, 16>(a, blocks, lds, stream);
}
