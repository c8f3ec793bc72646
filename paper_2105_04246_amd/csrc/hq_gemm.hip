// Gather-GEMM on int8 MFMA with the fused in-hindsight epilogue (gfx950).
//
// One kernel serves the forward pass and the input gradient of linear and convolution
// layers (paper Sec. 3.1).  Both are  out[m][n] = sum_{tap,c} A[pix(m,tap)][c] * Bw[n][tap][c]:
//   forward:  m = output pixel, A = X,  pix = (oh*stride - pad + r, ow*stride - pad + s)
//   dgrad:    m = input pixel,  A = dY, pix = ((h + pad - r)/stride, (w + pad - s)/stride)
//             where that division is exact and lands inside the output image.
// Taps without a source pixel are filled with A's zero-point code (real zero), so that the
// zero point leaves the sum as one term per output column: z_a * bsum[n].
//
// The accumulators never leave registers on the fused path (Sec. 3.2, static quantization):
// the epilogue removes the zero point, folds min / max / clip counts of the tile into the
// tensor's statistics (Sec. 4, step 2) and stores 8-bit codes quantized with the range that
// was fixed before the launch (Sec. 4, step 1).  With `out32` set instead, the same kernel is
// pass 1 of the dynamic baseline: it stores the corrected 32-bit outputs (eq. (5), "save
// acc output") and gathers min / max only.
#include "hq_device.h"

namespace {

constexpr int BK = 64;            // bytes of reduction staged per step (two MFMA k-steps of 32)
constexpr int PITCH = BK + 16;    // LDS row pitch: 80 B keeps 16-byte fragment reads conflict-free

struct GemmArgs {
    const int8_t *A, *Bw;
    const int32_t *bsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int M, N;                      // output rows (pixels) and columns (channels)
    int Cs;                        // reduced channels per tap
    int cpt;                       // 16-byte chunks per tap = ceil(Cs / 16)
    int nchunks;                   // taps * cpt
    int R, S;
    int Hs, Ws;                    // spatial size of the gathered tensor A
    int Ho, Wo;                    // spatial size the row index m runs over
    int stride, pad;
    int dgrad;                     // 0 forward gather, 1 input-gradient gather
    int aligned16;                 // Cs % 16 == 0: every chunk is one aligned 16-byte load
};

__device__ inline v4i load_chunk(const int8_t *p, int nbytes, bool aligned16, int fill)
{
    if (aligned16) return *reinterpret_cast<const v4i *>(p);
    v4i v;
    const int *q = reinterpret_cast<const int *>(p);
    v[0] = nbytes > 0 ? q[0] : fill;
    v[1] = nbytes > 4 ? q[1] : fill;
    v[2] = nbytes > 8 ? q[2] : fill;
    v[3] = nbytes > 12 ? q[3] : fill;
    return v;
}

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(HQ_THREADS) void hq_gemm_kernel(const GemmArgs a)
{
    static_assert(WGM * WGN == HQ_THREADS / 64, "four wavefronts");
    constexpr int WTM = BM / WGM, WTN = BN / WGN;      // wavefront tile
    constexpr int MT = WTM / 32, NT = WTN / 32;        // 32x32 MFMA tiles per wavefront
    constexpr int AROWS = BM / 64;                     // A rows loaded per thread per stage
    constexpr int BROWS = (BN + 63) / 64;              // B rows loaded per thread per stage

    __shared__ __attribute__((aligned(16))) int8_t As[2][BM * PITCH];
    __shared__ __attribute__((aligned(16))) int8_t Bs[2][BN * PITCH];
    __shared__ int red[4 * (HQ_THREADS / 64)];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int n_tiles = (a.N + BN - 1) / BN;
    const int tile_m = blockIdx.x / n_tiles, tile_n = blockIdx.x % n_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int za = a.aq->zero_point;
    const int fill = (za & 0xff) * 0x01010101;

    // ---- per-thread gather state: AROWS rows of the A tile, one 16-byte column of them
    const int cc = tid & 3;                 // chunk column inside the 64-byte stage
    const int8_t *abase[AROWS];
    int ay[AROWS], ax[AROWS];
    bool arow_ok[AROWS];
#pragma unroll
    for (int i = 0; i < AROWS; i++) {
        int m = m0 + (tid >> 2) + 64 * i;
        arow_ok[i] = m < a.M;
        int mm = arow_ok[i] ? m : 0;
        int x = mm % a.Wo, y = (mm / a.Wo) % a.Ho, b = mm / (a.Wo * a.Ho);
        abase[i] = a.A + (size_t)b * a.Hs * a.Ws * a.Cs;
        ay[i] = a.dgrad ? y + a.pad : y * a.stride - a.pad;
        ax[i] = a.dgrad ? x + a.pad : x * a.stride - a.pad;
    }
    const size_t brow_len = (size_t)a.R * a.S * a.Cs;      // bytes per weight row
    // chunk cursor (same for A and B): chunk index -> (r, s, c16)
    int chunk = cc, c16 = cc % a.cpt, tap = cc / a.cpt;
    int tr = tap / a.S, ts = tap % a.S;

    v4i areg[AROWS], breg[BROWS];
    auto load_stage = [&]() {
        const bool chunk_ok = chunk < a.nchunks;
        const int coff = c16 * 16, nbytes = a.Cs - coff;
#pragma unroll
        for (int i = 0; i < AROWS; i++) {
            int iy, ix; bool ok = chunk_ok && arow_ok[i];
            if (!a.dgrad) {
                iy = ay[i] + tr; ix = ax[i] + ts;
            } else {
                iy = ay[i] - tr; ix = ax[i] - ts;
                if (a.stride != 1) {
                    ok = ok && iy >= 0 && ix >= 0 && (iy % a.stride == 0) && (ix % a.stride == 0);
                    iy /= a.stride; ix /= a.stride;
                }
            }
            ok = ok && iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws;
            v4i v = {fill, fill, fill, fill};
            if (ok) v = load_chunk(abase[i] + ((size_t)iy * a.Ws + ix) * a.Cs + coff, nbytes, a.aligned16, fill);
            areg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BROWS; i++) {
            int row = (tid >> 2) + 64 * i, n = n0 + row;
            v4i v = {0, 0, 0, 0};
            if (row < BN && n < a.N && chunk_ok)
                v = load_chunk(a.Bw + (size_t)n * brow_len + (size_t)tap * a.Cs + coff, nbytes, a.aligned16, 0);
            breg[i] = v;
        }
        // advance the cursor by one stage (4 chunks)
        chunk += 4; c16 += 4;
        while (c16 >= a.cpt) { c16 -= a.cpt; tap++; ts++; if (ts == a.S) { ts = 0; tr++; } }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < AROWS; i++)
            *reinterpret_cast<v4i *>(&As[buf][((tid >> 2) + 64 * i) * PITCH + cc * 16]) = areg[i];
#pragma unroll
        for (int i = 0; i < BROWS; i++) {
            int row = (tid >> 2) + 64 * i;
            if (row < BN) *reinterpret_cast<v4i *>(&Bs[buf][row * PITCH + cc * 16]) = breg[i];
        }
    };

    v16i acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0;

    const int KT = (a.nchunks + 3) / 4;
    load_stage();
    store_stage(0);
    __syncthreads();
    const int frag_off = (lane & 31) * PITCH + (lane >> 5) * 16;
    for (int kt = 0; kt < KT; kt++) {
        const int buf = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) load_stage();
        const int ksteps = min(4, a.nchunks - 4 * kt) > 2 ? 2 : 1;
        for (int ks = 0; ks < ksteps; ks++) {
            v4i wf[NT], af[MT];
#pragma unroll
            for (int j = 0; j < NT; j++)
                wf[j] = *reinterpret_cast<const v4i *>(&Bs[buf][(wn * WTN + j * 32) * PITCH + frag_off + ks * 32]);
#pragma unroll
            for (int i = 0; i < MT; i++)
                af[i] = *reinterpret_cast<const v4i *>(&As[buf][(wm * WTM + i * 32) * PITCH + frag_off + ks * 32]);
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], acc[i][j], 0, 0, 0);
        }
        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  With weights as the first MFMA operand, lane l holds output row
    // (l % 32) of the tile and, for register r, column 8*(r/4) + 4*(l/32) + r%4: four
    // consecutive output channels per register quad, i.e. one 32-bit store of codes.
    const bool fused = a.out32 == nullptr;
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqRequant rq = {1.0f, 0.0f, 0.0f, 0};
    if (fused) rq = hq_make_requant(acc_scale, a.range->qp, a.range->qlo, a.range->qhi);
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;
#pragma unroll
    for (int i = 0; i < MT; i++) {
        const int m = m0 + wm * WTM + i * 32 + (lane & 31);
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < NT; j++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int n = n0 + wn * WTN + j * 32 + 8 * g + 4 * (lane >> 5);
                if (n >= a.N) continue;
                const v4i bs = *reinterpret_cast<const v4i *>(a.bsum + n);
                int c[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    c[e] = acc[i][j][4 * g + e] - za * bs[e];
                    mn = min(mn, c[e]); mx = max(mx, c[e]);
                }
                if (fused) {
                    int q[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) q[e] = hq_requant(c[e], rq, nlo, nhi);
                    *reinterpret_cast<unsigned *>(a.out8 + (size_t)m * a.N + n) = hq_pack4(q[0], q[1], q[2], q[3]);
                } else {
                    v4i v = {c[0], c[1], c[2], c[3]};
                    *reinterpret_cast<v4i *>(a.out32 + (size_t)m * a.N + n) = v;
                }
            }
        }
    }
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.N);
        if (fused) *a.outq = a.range->qp;
    }
}

template <int BM, int BN, int WGM, int WGN>
int launch(const GemmArgs &a, hipStream_t s)
{
    const long tiles = (long)((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL((hq_gemm_kernel<BM, BN, WGM, WGN>), dim3((unsigned)tiles), dim3(HQ_THREADS), 0, s, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

} // namespace

// Host-side entry used by hq_api.hip.  `dgrad` selects the gather; `out32` the dynamic pass 1.
int hq_launch_gemm(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                   const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                   int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream)
{
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    GemmArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.R = p->R; a.S = p->S; a.stride = p->stride; a.pad = p->pad; a.dgrad = dgrad;
    if (!dgrad) {
        a.M = p->B * OH * OW; a.N = p->Cout; a.Cs = p->C;
        a.Hs = p->H; a.Ws = p->W; a.Ho = OH; a.Wo = OW;
    } else {
        a.M = p->B * p->H * p->W; a.N = p->C; a.Cs = p->Cout;
        a.Hs = OH; a.Ws = OW; a.Ho = p->H; a.Wo = p->W;
    }
    a.cpt = (a.Cs + 15) / 16;
    a.nchunks = p->R * p->S * a.cpt;
    a.aligned16 = (a.Cs % 16) == 0;
    if (a.N > 64) return launch<128, 128, 2, 2>(a, stream);
    if (a.N > 32) return launch<256, 64, 4, 1>(a, stream);
    return launch<256, 32, 4, 1>(a, stream);
}
