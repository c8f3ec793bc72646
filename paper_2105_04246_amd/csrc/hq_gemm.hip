// Gather-GEMM on int8 MFMA with the fused in-hindsight epilogue (gfx950): the general path of
// hq_gemm_fwd / hq_gemm_dgrad and of pass 1 of the dynamic baseline, for every supported
// shape that the weights-resident kernel does not take (large channel counts, linear layers,
// strided input gradients, channel counts that are not multiples of 16).
//
// Both operations are  out[m][n] = sum_{tap,c} A[pix(m,tap)][c] * Bw[n][tap][c]   (paper Sec. 3.1):
//   forward:            m = output pixel, A = X,  pix = (oh*stride - pad + r, ow*stride - pad + s)
//   dgrad, stride 1:    the same stencil over dY with padding R-1-pad and mirrored taps
//   dgrad, stride > 1:  m = input pixel, A = dY, pix = ((h + pad - r)/stride, (w + pad - s)/stride)
//                       where the division is exact and lands inside the output image.  With
//                       16-byte-aligned channel counts the input pixels are split into the
//                       stride^2 classes (h % stride, w % stride): inside a class only the taps
//                       r = r0 + stride*jr, s = s0 + stride*js ever divide exactly, and the class
//                       is a stride-1 stencil over dY with those taps.  A tile holds pixels of one
//                       class and reduces over that class's taps only.
// Taps without a source pixel are filled with A's zero-point code (real zero), so the zero
// point leaves the sum as one term per output column, z_a * bsum[n].
//
// Tiling: 256 threads (2x2 or 4x1 wavefronts), v_mfma_i32_32x32x32_i8, weights as the first
// operand.  Weight rows are stored in LDS in a permuted order so that a lane ends up with 16
// consecutive output channels of one pixel (one 16-byte store).  K is staged through LDS
// (two buffers, the next stage's global loads in flight during the current stage's MFMAs),
// rows padded by 16 bytes to keep 16-byte fragment reads free of bank conflicts.  Tiles that
// share their A rows (same pixels, different channel blocks) get consecutive slots on the
// same XCD, so the second reader finds the rows in that XCD's L2 (except in the class form, whose
// tiles differ in work from class to class and are dealt round-robin; a class without taps is
// filled with the zero-point code and leaves).  Tile shapes: 128x128, 256x64, 256x32, and
// 64x64 for launches that 128x128 tiles would leave with fewer workgroups than compute units.
//
// The accumulators never leave registers on the fused path (Sec. 3.2, static quantization):
// the epilogue removes the zero point, folds min / max / clip counts into the tensor's
// statistics (Sec. 4, step 2) and stores codes quantized with the range fixed before the
// launch (Sec. 4, step 1).  With `out32` set, the kernel is pass 1 of the dynamic baseline:
// it stores the corrected 32-bit outputs (the accumulator-save term of eq. (5)) and gathers min / max.
#include "hq_device.h"
#include <type_traits>

namespace {

// 16-byte rows of one repeated byte value, indexed by that value: the source of the lanes of a direct-to-LDS
// load that have no source of their own (padding taps: zero-point code; rows and chunks past the end: 0), so
// that a stage's loads need no branch per row.
struct GemmFillRows {
    unsigned w[256][4];
    constexpr GemmFillRows() : w()
    {
        for (int v = 0; v < 256; v++)
            for (int k = 0; k < 4; k++) w[v][k] = (unsigned)v * 0x01010101u;
    }
};
__device__ const GemmFillRows gemm_fill_rows = GemmFillRows();

// Class form of a strided input gradient: output pixels with (y mod stride, x mod stride) = (ph, pw) see the
// same taps; such a class is an image of Hc x Wc pixels under a stride-1 stencil of nr x ns taps.
struct GemmClass {
    int ph, pw, Hc, Wc;
    int r0, s0, nr, ns;            // first filter row / column the class sees, and how many (every stride-th)
    int dh, dw;                    // offset of the class's pixel (y, x) into the gathered tensor
    unsigned magic_Wc, magic_Hc;   // ceil(2^32 / d)
};

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
    int cpt;                       // aligned: 16-byte chunks per tap = Cs / 16
    int nchunks;                   // 16-byte chunks of the reduction: taps * cpt, or ceil(taps * Cs / 16)
    int kcols;                     // taps * Cs
    unsigned magic_Cs, magic_S;    // for hq_magic_div
    int taps, S;
    int Hs, Ws;                    // spatial size of the gathered tensor A
    int Ho, Wo;                    // spatial size the row index m runs over
    int stride, pad;               // stencil form: effective stride / padding
    int flip;                      // weight taps mirrored (dgrad written as a stencil)
    int m_tiles, n_tiles;
    int Bn;                        // images (class form)
    int ncls;                      // class form: stride * stride classes, 0 otherwise
    int cls_tile0[17];             // first row tile of each class (prefix sums), [ncls] = m_tiles
    GemmClass cls[16];             // class form: the stencil of every class, worked out once on the host
    unsigned magic_Wo, magic_Ho;   // ceil(2^32 / d) for the pixel decode (hq_magic_div)
    int magic_ok;                  // the decode's operands are in hq_magic_div's range; 0: plain division
    HqSr sr;                       // MODE 2: seed of the stochastic rounding
};

__device__ inline int sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

// BKB: bytes of reduction per stage.  STRIDED: input gradient of a strided layer (gather with
// exact-division test); otherwise the stencil form.  ALIGNED: Cs % 16 == 0 (16-byte loads, one tap per chunk).
// MODE 0: 32-bit outputs (pass 1 of the dynamic baseline); 1: requantize, round to nearest even; 2: requantize,
// stochastic rounding.
template <int BM, int BN, int WGM, int WGN, int BKB, bool STRIDED, bool ALIGNED, int MODE>
__global__ __launch_bounds__(HQ_THREADS, (BKB == 64 && BM == 128 && ALIGNED ? 4 : 2)) void hq_gemm_kernel(const GemmArgs a)
{
    static_assert(WGM * WGN == HQ_THREADS / 64, "four wavefronts");
    constexpr bool FUSED = MODE != 0, SR = MODE == 2;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;       // wavefront tile
    constexpr int MT = WTM / 32, NT = WTN / 32;         // 32x32 MFMA tiles per wavefront
    constexpr int CPS = BKB / 16;                       // 16-byte chunks per row and stage
    constexpr int RPP = HQ_THREADS / CPS;               // rows covered by one pass of the loader
    constexpr int AROWS = BM / RPP, BROWS = (BN + RPP - 1) / RPP;
    constexpr int PITCH = ALIGNED ? BKB : BKB + 16;     // aligned: dense rows, 16-byte chunks XOR-swizzled
    constexpr int KS = BKB / 32;

    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t *As = smem;                                   // [2][BM][PITCH]
    int8_t *Bs = smem + 2 * BM * PITCH;                  // [2][BN][PITCH]
    int *bzs = reinterpret_cast<int *>(smem + 2 * (BM + BN) * PITCH);      // [BN] z_a * bsum[n0 + col]
    int *red = bzs + BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // tile of this workgroup: ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous run of tiles (channel blocks of one pixel block next to each other)
    // (not in the class form of a strided input gradient: its classes are runs of row tiles with
    // different numbers of taps, down to none, and a contiguous run per XCD would leave the heavy
    // classes to one or two XCDs)
    int tile = blockIdx.x;
    if (!(STRIDED && ALIGNED)) {
        const int total = a.m_tiles * a.n_tiles, per = total / 8;
        if (per > 0 && tile < per * 8) tile = (tile & 7) * per + (tile >> 3);
    }
    int tile_m = tile / a.n_tiles;
    const int tile_n = tile - tile_m * a.n_tiles;
    const int n0 = tile_n * BN;

    // class form (strided input gradient): the tile's class and that class's stencil
    constexpr bool CLASSED = STRIDED && ALIGNED;
    int Hc = a.Ho, Wc = a.Wo, Mrows = a.M, ph = 0, pw = 0, r0 = 0, s0 = 0, nr = 0, ns = 1, dh = 0, dw = 0;
    int nchunks = a.nchunks;
    unsigned mWc = a.magic_Wo, mHc = a.magic_Ho;
    if (CLASSED) {
        int cls = 0;
        while (cls + 1 < a.ncls && tile_m >= a.cls_tile0[cls + 1]) cls++;
        tile_m -= a.cls_tile0[cls];
        const GemmClass &g = a.cls[cls];
        ph = g.ph; pw = g.pw; Hc = g.Hc; Wc = g.Wc; r0 = g.r0; s0 = g.s0; nr = g.nr; ns = g.ns; dh = g.dh; dw = g.dw;
        mWc = g.magic_Wc; mHc = g.magic_Hc;
        Mrows = a.Bn * Hc * Wc;
        nchunks = nr * ns * a.cpt;
        if (ns == 0) ns = 1;                       // no taps at all: nchunks == 0, nothing is decoded
    }
    const int m0 = tile_m * BM;
    // row of the tile's image grid -> (x, y, image): two reciprocal multiplications (a division costs some 40
    // instructions, and short reductions have few MFMAs to hide them behind)
    auto decode = [&](int m, int &x, int &y, int &b) {
        if (a.magic_ok) {
            const unsigned t = hq_magic_div((unsigned)m, mWc), bb = hq_magic_div(t, mHc);
            x = (int)((unsigned)m - t * (unsigned)Wc); y = (int)(t - bb * (unsigned)Hc); b = (int)bb;
        } else {
            x = m % Wc; const int t = m / Wc; y = t % Hc; b = t / Hc;
        }
    };

    if (CLASSED && nchunks == 0) {
        // A class no filter tap reaches (1x1 filters with stride 2: three of the four classes): every
        // output of the tile is real zero, its code the zero point.  Stored directly, a row's columns by
        // neighbouring lanes, instead of going through the tile machinery.
        const int cols = min(BN, a.N - n0);                 // multiple of 4
        const bool wide = ((cols | a.N) & 15) == 0;         // 16-byte pieces, else 4-byte ones
        const int ppr = wide ? cols / 16 : cols / 4;        // pieces per row (at most 32)
        const int rpp = HQ_THREADS / ppr;                   // rows per pass of the workgroup
        const int rl = tid / ppr, piece = tid - rl * ppr;
        const int zcode = a.range->qp.zero_point & 0xff;    // inside the grid by construction
        const int fillw = (int)((unsigned)zcode * 0x01010101u);
        if (rl < rpp) {
            // the row's pixel is decoded once and then stepped (rpp rows per pass)
            int m = m0 + rl;
            int x, y, b;
            decode(m, x, y, b);
            for (int row = rl; row < BM && m < Mrows; row += rpp, m += rpp) {
                const size_t px = (size_t)(b * a.Ho + ph + a.stride * y) * a.Wo + pw + a.stride * x;
                const size_t o = px * a.N + n0;
                if (MODE == 0) {
                    const v4i z4 = {0, 0, 0, 0};
                    for (int q = 0; q < (wide ? 4 : 1); q++)
                        *reinterpret_cast<v4i *>(a.out32 + o + (wide ? 16 * piece + 4 * q : 4 * piece)) = z4;
                } else if (wide) {
                    const v4i f4 = {fillw, fillw, fillw, fillw};
                    *reinterpret_cast<v4i *>(a.out8 + o + 16 * piece) = f4;
                } else {
                    *reinterpret_cast<int *>(a.out8 + o + 4 * piece) = fillw;
                }
                x += rpp;
                while (x >= Wc) { x -= Wc; if (++y == Hc) { y = 0; b++; } }
            }
        }
        int *red0 = reinterpret_cast<int *>(smem);
        hq_block_stats_commit(0, 0, 0, 0, a.st, red0);      // the accumulators of this tile are all 0
        if (blockIdx.x == 0 && tid == 0) {
            a.st->acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
            atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.N);
            if (MODE != 0) *a.outq = a.range->qp;
        }
        return;
    }

    const int za = a.aq->zero_point;
    const int fill = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31

    // z_a * (sum of the weights the reduction runs over), visible after the first barrier
    if (tid < BN) {
        int bz = 0;
        const int n = n0 + tid;
        if (n < a.N) {
            if (!CLASSED) {
                bz = za * a.bsum[n];
            } else if (za != 0) {
                int sum = 0;
                for (int jr = 0; jr < nr; jr++)
                    for (int js = 0; js * a.stride + s0 < a.S; js++) {
                        const int8_t *w = a.Bw + ((size_t)n * a.taps + (r0 + a.stride * jr) * a.S + s0 + a.stride * js) * a.Cs;
                        for (int k = 0; k < a.Cs; k += 16) {
                            const v4i v = *reinterpret_cast<const v4i *>(w + k);
#pragma unroll
                            for (int d = 0; d < 4; d++) sum = __builtin_amdgcn_sdot4(v[d], 0x01010101, sum, false);
                        }
                    }
                bz = za * sum;
            }
        }
        bzs[tid] = bz;
    }

    // ---- per-thread gather state
    const int cc = tid % CPS, lrow = tid / CPS;
    const int8_t *abase[AROWS];
    int ay[AROWS], ax[AROWS];
    bool arow_ok[AROWS];
#pragma unroll
    for (int i = 0; i < AROWS; i++) {
        const int m = m0 + lrow + RPP * i;
        arow_ok[i] = m < Mrows;
        const int mm = arow_ok[i] ? m : 0;
        int x, y, b;
        decode(mm, x, y, b);
        abase[i] = a.A + (size_t)b * a.Hs * a.Ws * a.Cs;
        ay[i] = CLASSED ? y + dh : STRIDED ? y + a.pad : y * a.stride - a.pad;
        ax[i] = CLASSED ? x + dw : STRIDED ? x + a.pad : x * a.stride - a.pad;
    }
    // Aligned form: per row, the address of tap (0, 0) and a bit per tap that says whether the tap has a
    // source pixel, so that a stage costs one 64-bit add and one bit test per row instead of the
    // bounds arithmetic and a 64-bit multiply (up to 64 taps; larger filters test bounds per stage).
    const int taps_eff = CLASSED ? nr * ns : a.taps, tapw_eff = CLASSED ? ns : a.S;
    const bool use_mask = ALIGNED && taps_eff <= 64;
    const int8_t *arow[AROWS];
    unsigned long long amask[AROWS];
    if (ALIGNED) {
#pragma unroll
        for (int i = 0; i < AROWS; i++) {
            arow[i] = abase[i] + ((ptrdiff_t)ay[i] * a.Ws + ax[i]) * a.Cs;
            unsigned long long mk = 0;
            if (use_mask && arow_ok[i]) {
                for (int t = 0, r = 0, c = 0; t < taps_eff; t++, c++) {
                    if (c == tapw_eff) { c = 0; r++; }
                    const int iy = CLASSED ? ay[i] - r : ay[i] + r, ix = CLASSED ? ax[i] - c : ax[i] + c;
                    if (iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws) mk |= 1ull << t;
                }
            }
            amask[i] = mk;
        }
    }
    const int8_t *bbase[BROWS];
    bool brow_ok[BROWS];
    const size_t brow_len = (size_t)a.taps * a.Cs;
#pragma unroll
    for (int i = 0; i < BROWS; i++) {
        const int row = lrow + RPP * i;                   // LDS row; holds channel sigma-permuted in its 32-block
        const int n = n0 + (row & ~31) + sigma32(row & 31);
        brow_ok[i] = row < BN && n < a.N;
        bbase[i] = a.Bw + (size_t)(brow_ok[i] ? n : 0) * brow_len;
    }
    // Aligned form: rows are dense in LDS and the 16-byte chunks of a row are XOR-swizzled by the row
    // index, which keeps the fragment reads free of bank conflicts without padding.  The LDS slot of
    // a thread is fixed (slot = thread: that is where a direct-to-LDS load of lane l lands), so the
    // swizzle is applied to the chunk the thread fetches instead.
    auto swz = [](int row) { return CPS == 8 ? ((row >> 1) & 7) : ((row >> 2) & (CPS - 1)); };
    const int csrc = ALIGNED ? (cc ^ swz(lrow)) : cc;
    const int tapw = CLASSED ? ns : a.S;             // taps per row of the tap grid the chunks run over
    int chunk = csrc, c16 = csrc, tap = 0, tr = 0, ts = 0;       // csrc < CPS: a few subtractions instead of divisions
    while (c16 >= a.cpt) { c16 -= a.cpt; tap++; if (++ts == tapw) { ts = 0; tr++; } }


    // Aligned form: global -> LDS without passing through registers (global_load_lds_dwordx4: lane l
    // of a wavefront writes 16 bytes at base + 16 * l).  Lanes without a source (padding taps, rows
    // past the end, chunks past the end of K) read a row of the fill table instead: no branch per row.
    auto issue_stage = [&](int buf) {
        const bool chunk_ok = chunk < nchunks;
        const int coff = c16 * 16;
        const int8_t *fill_src = reinterpret_cast<const int8_t *>(gemm_fill_rows.w[za & 0xff]);
        const int8_t *zero_src = reinterpret_cast<const int8_t *>(gemm_fill_rows.w[0]);
        const int tapoff = (CLASSED ? -(tr * a.Ws + ts) : tr * a.Ws + ts) * a.Cs + coff;   // from the row's tap (0, 0)
#pragma unroll
        for (int i = 0; i < AROWS; i++) {
            bool ok;
            if (use_mask) {
                ok = chunk_ok && ((amask[i] >> (tap & 63)) & 1ull) != 0;
            } else {
                const int iy = CLASSED ? ay[i] - tr : ay[i] + tr, ix = CLASSED ? ax[i] - ts : ax[i] + ts;
                ok = chunk_ok && arow_ok[i] && iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws;
            }
            int8_t *dst = As + (size_t)buf * BM * BKB + 4096 * i + (tid & ~63) * 16;      // this wavefront's 1 KiB
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ok ? arow[i] + tapoff : fill_src),
                                             (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
        }
        const int wtap = CLASSED ? (r0 + a.stride * tr) * a.S + s0 + a.stride * ts : a.flip ? a.taps - 1 - tap : tap;
#pragma unroll
        for (int i = 0; i < BROWS; i++) {
            if (lrow + RPP * i < BN) {
                int8_t *dst = Bs + (size_t)buf * BN * BKB + 4096 * i + (tid & ~63) * 16;
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(brow_ok[i] && chunk_ok ? bbase[i] + (size_t)wtap * a.Cs + coff : zero_src),
                    (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
            }
        }
        chunk += CPS; c16 += CPS;
        while (c16 >= a.cpt) { c16 -= a.cpt; tap++; ts++; if (ts == tapw) { ts = 0; tr++; } }
    };

    v4i areg0[AROWS], breg0[BROWS], areg1[AROWS], breg1[BROWS];
    auto load_stage = [&](v4i (&areg)[AROWS], v4i (&breg)[BROWS]) {
        {
            // Channel counts that are not multiples of 16: the reduction runs over the (tap, channel)
            // pairs as they lie in a weight row, 4 bytes at a time (a 4-byte word never straddles two
            // taps because Cs % 4 == 0), so a tap costs Cs bytes of the reduction, not a padded 16.
            int dr[4], ds[4], doff[4], dw[4];
            bool dok[4];
#pragma unroll
            for (int d = 0; d < 4; d++) {
                const int kc = chunk * 16 + 4 * d;
                dok[d] = kc < a.kcols;
                const int t = (int)hq_magic_div((unsigned)kc, a.magic_Cs), cx = kc - t * a.Cs;
                dr[d] = (int)hq_magic_div((unsigned)t, a.magic_S); ds[d] = t - dr[d] * a.S;
                doff[d] = cx;
                dw[d] = (a.flip ? a.taps - 1 - t : t) * a.Cs + cx;
            }
#pragma unroll
            for (int i = 0; i < AROWS; i++) {
                v4i v = {fill, fill, fill, fill};
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    int iy, ix;
                    bool ok = dok[d] && arow_ok[i];
                    if (!STRIDED) {
                        iy = ay[i] + dr[d]; ix = ax[i] + ds[d];
                    } else {
                        iy = ay[i] - dr[d]; ix = ax[i] - ds[d];
                        ok = ok && iy >= 0 && ix >= 0 && (iy % a.stride == 0) && (ix % a.stride == 0);
                        iy /= a.stride; ix /= a.stride;
                    }
                    ok = ok && iy >= 0 && iy < a.Hs && ix >= 0 && ix < a.Ws;
                    if (ok) v[d] = *reinterpret_cast<const int *>(abase[i] + ((size_t)iy * a.Ws + ix) * a.Cs + doff[d]);
                }
                areg[i] = v;
            }
#pragma unroll
            for (int i = 0; i < BROWS; i++) {
                v4i v = {0, 0, 0, 0};
#pragma unroll
                for (int d = 0; d < 4; d++)
                    if (brow_ok[i] && dok[d]) v[d] = *reinterpret_cast<const int *>(bbase[i] + dw[d]);
                breg[i] = v;
            }
            chunk += CPS;
        }
    };
    auto store_stage = [&](int buf, const v4i (&areg)[AROWS], const v4i (&breg)[BROWS]) {
#pragma unroll
        for (int i = 0; i < AROWS; i++)
            *reinterpret_cast<v4i *>(As + (buf * BM + lrow + RPP * i) * PITCH + cc * 16) = areg[i];
#pragma unroll
        for (int i = 0; i < BROWS; i++)
            if (lrow + RPP * i < BN)
                *reinterpret_cast<v4i *>(Bs + (buf * BN + lrow + RPP * i) * PITCH + cc * 16) = breg[i];
    };

    v16i acc[MT][NT];

    // K loop.  Two LDS buffers and two register sets: while stage kt is multiplied from LDS, the
    // global loads of stage kt+2 are in flight and stage kt+1 waits in registers, so a load has
    // two stages of MFMA work to hide behind.
    const int KT = (nchunks + CPS - 1) / CPS;
    int frag_off[KS];                                     // lane's 16 bytes of k-step ks inside its row block
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
        frag_off[ks] = (lane & 31) * PITCH + 16 * (ALIGNED ? ((2 * ks + (lane >> 5)) ^ swz(lane & 31)) : 2 * ks + (lane >> 5));
    auto compute = [&](int buf) {
        const int8_t *Ab = As + (buf * BM + wm * WTM) * PITCH;
        const int8_t *Bb = Bs + (buf * BN + wn * WTN) * PITCH;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {                 // chunks past the end of K hold zero weights
            v4i wf[NT], af[MT];
#pragma unroll
            for (int j = 0; j < NT; j++) wf[j] = *reinterpret_cast<const v4i *>(Bb + j * 32 * PITCH + frag_off[ks]);
#pragma unroll
            for (int i = 0; i < MT; i++) af[i] = *reinterpret_cast<const v4i *>(Ab + i * 32 * PITCH + frag_off[ks]);
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], acc[i][j], 0, 0, 0);
        }
    };
    if constexpr (ALIGNED) {
        issue_stage(0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        load_stage(areg0, breg0);
        store_stage(0, areg0, breg0);
        if (KT > 1) load_stage(areg1, breg1);
    }
    __syncthreads();
    // the accumulators start at -z_a * bsum[n]: the zero-point term of the sum is gone before
    // the epilogue looks at them (lane = 16 consecutive channels of column block j)
#pragma unroll
    for (int j = 0; j < NT; j++) {
        const int cb = wn * WTN + j * 32 + 16 * (lane >> 5);
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const v4i bz = *reinterpret_cast<const v4i *>(bzs + cb + 4 * g);
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int e = 0; e < 4; e++) acc[i][j][4 * g + e] = -bz[e];
        }
    }
    if constexpr (ALIGNED) {
        // stage kt+1 lands in the other buffer while stage kt is multiplied
        for (int kt = 0; kt < KT; kt++) {
            if (kt + 1 < KT) issue_stage((kt + 1) & 1);
            compute(kt & 1);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    } else {
        for (int kt = 0; kt < KT; kt += 2) {
            if (kt + 2 < KT) load_stage(areg0, breg0);        // stage kt+2
            compute(0);
            if (kt + 1 < KT) store_stage(1, areg1, breg1);    // stage kt+1
            __syncthreads();
            if (kt + 1 < KT) {
                if (kt + 3 < KT) load_stage(areg1, breg1);    // stage kt+3
                compute(1);
                if (kt + 2 < KT) store_stage(0, areg0, breg0);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: lane = one pixel of a 32-row block, 16 consecutive channels per column block
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);
    const bool wide_store = (a.N & 15) == 0;
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;
    auto epilogue = [&](auto full) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int i = 0; i < MT; i++) {
            int m = m0 + wm * WTM + i * 32 + (lane & 31);
            if (m >= Mrows) continue;
            if (CLASSED) {                                  // row inside the class -> input pixel
                int x, y, b;
                decode(m, x, y, b);
                m = (b * a.Ho + ph + a.stride * y) * a.Wo + pw + a.stride * x;
            }
#pragma unroll
            for (int j = 0; j < NT; j++) {
                const int nb = n0 + wn * WTN + j * 32 + 16 * (lane >> 5);
                if (nb >= a.N) continue;
                int c[16];
#pragma unroll
                for (int r = 0; r < 16; r++) c[r] = acc[i][j][r];
                const size_t o = (size_t)m * a.N + nb;
                if (!FUSED) {
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        if (nb + 4 * g >= a.N) continue;       // N % 4 == 0: a quad is all in or all out
                        hq_minmax_group<4>(c + 4 * g, mn, mx);
                        const v4i v = {c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                        *reinterpret_cast<v4i *>(a.out32 + o + 4 * g) = v;
                    }
                } else if (nb + 16 <= a.N) {
                    int w[4];
                    if (SR) hq_requant_group_sr<16, FULL>(c, ep, a.sr, o, mn, mx, nlo, nhi, w);
                    else    hq_requant_group<16, FULL>(c, ep, mn, mx, nlo, nhi, w);
                    if (wide_store) {
                        const v4i v = {w[0], w[1], w[2], w[3]};
                        *reinterpret_cast<v4i *>(a.out8 + o) = v;
                    } else {
#pragma unroll
                        for (int g = 0; g < 4; g++) *reinterpret_cast<int *>(a.out8 + o + 4 * g) = w[g];
                    }
                } else {
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        if (nb + 4 * g >= a.N) continue;
                        int w;
                        if (SR) hq_requant_group_sr<4, FULL>(c + 4 * g, ep, a.sr, o + 4 * g, mn, mx, nlo, nhi, &w);
                        else    hq_requant_group<4, FULL>(c + 4 * g, ep, mn, mx, nlo, nhi, &w);
                        *reinterpret_cast<int *>(a.out8 + o + 4 * g) = w;
                    }
                }
            }
        }
    };
    if (ep.full_grid) epilogue(std::true_type()); else epilogue(std::false_type());
    __syncthreads();
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, (unsigned long long)a.M * (unsigned long long)a.N);
        if (FUSED) *a.outq = a.range->qp;
    }
}

template <int BM, int BN, int WGM, int WGN, int BKB, bool STRIDED, bool ALIGNED, int MODE>
int launch3(GemmArgs &a, hipStream_t s)
{
    a.m_tiles = (a.M + BM - 1) / BM;
    a.n_tiles = (a.N + BN - 1) / BN;
    a.ncls = 0;
    a.magic_ok = (unsigned long long)a.M * (unsigned long long)(a.Wo > a.Ho ? a.Wo : a.Ho) < (1ull << 32);
    a.magic_Wo = hq_magic32((unsigned)a.Wo);
    a.magic_Ho = hq_magic32((unsigned)a.Ho);
    if (STRIDED && ALIGNED) {
        a.ncls = a.stride * a.stride;
        int t = 0;
        for (int c = 0; c < a.ncls; c++) {
            const int ph = c / a.stride, pw = c % a.stride;
            const int Hc = (a.Ho - ph + a.stride - 1) / a.stride, Wc = (a.Wo - pw + a.stride - 1) / a.stride;
            GemmClass &g = a.cls[c];
            g.ph = ph; g.pw = pw; g.Hc = Hc; g.Wc = Wc;
            g.r0 = (ph + a.pad) % a.stride; g.s0 = (pw + a.pad) % a.stride;
            const int R = a.taps / a.S;
            g.nr = g.r0 < R ? (R - g.r0 + a.stride - 1) / a.stride : 0;
            g.ns = g.s0 < a.S ? (a.S - g.s0 + a.stride - 1) / a.stride : 0;
            g.dh = (ph + a.pad - g.r0) / a.stride; g.dw = (pw + a.pad - g.s0) / a.stride;
            g.magic_Wc = Wc > 0 ? hq_magic32((unsigned)Wc) : 0u;
            g.magic_Hc = Hc > 0 ? hq_magic32((unsigned)Hc) : 0u;
            a.cls_tile0[c] = t;
            t += (a.Bn * Hc * Wc + BM - 1) / BM;
        }
        a.cls_tile0[a.ncls] = t;
        a.m_tiles = t;
    }
    const size_t lds = 2 * (size_t)(BM + BN) * (ALIGNED ? BKB : BKB + 16) + 4 * BN + 64;
    auto kern = hq_gemm_kernel<BM, BN, WGM, WGN, BKB, STRIDED, ALIGNED, MODE>;
    static bool configured = false;
    if (!configured) {
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return HQ_E_HIP;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.m_tiles * a.n_tiles)), dim3(HQ_THREADS), lds, s, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

// mode: 0 / 1 / 2 as the kernel's MODE.  Stochastic rounding is built for the two tile shapes with 64-byte
// stages only (the launcher below routes it there).
template <int BM, int BN, int WGM, int WGN, int BKB, bool STRIDED, bool ALIGNED>
int launch2m(GemmArgs &a, int mode, hipStream_t s)
{
    if (mode == 0) return launch3<BM, BN, WGM, WGN, BKB, STRIDED, ALIGNED, 0>(a, s);
    if (mode == 1) return launch3<BM, BN, WGM, WGN, BKB, STRIDED, ALIGNED, 1>(a, s);
    if constexpr (BKB == 64 && BN >= 64) return launch3<BM, BN, WGM, WGN, BKB, STRIDED, ALIGNED, 2>(a, s);
    return HQ_E_BADSHAPE;
}

template <int BM, int BN, int WGM, int WGN, int BKB>
int launch2(GemmArgs &a, bool strided, bool aligned, int mode, hipStream_t s)
{
    if (strided) {
        if (aligned) return launch2m<BM, BN, WGM, WGN, BKB, true, true>(a, mode, s);
        return launch2m<BM, BN, WGM, WGN, BKB, true, false>(a, mode, s);
    }
    if (aligned) return launch2m<BM, BN, WGM, WGN, BKB, false, true>(a, mode, s);
    return launch2m<BM, BN, WGM, WGN, BKB, false, false>(a, mode, s);
}

} // namespace

// Host-side entry used by hq_api.hip.  `dgrad` selects the operation; `out32` the dynamic pass 1.
int hq_launch_gemm(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                   const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                   int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed)
{
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    GemmArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.taps = p->R * p->S; a.S = p->S; a.Bn = p->B;
    bool strided = false;
    if (!dgrad) {
        a.M = p->B * OH * OW; a.N = p->Cout; a.Cs = p->C;
        a.Hs = p->H; a.Ws = p->W; a.Ho = OH; a.Wo = OW;
        a.stride = p->stride; a.pad = p->pad; a.flip = 0;
    } else {
        a.M = p->B * p->H * p->W; a.N = p->C; a.Cs = p->Cout;
        a.Hs = OH; a.Ws = OW; a.Ho = p->H; a.Wo = p->W;
        if (p->stride == 1 && p->R == p->S) {             // stencil over dY with mirrored taps
            a.stride = 1; a.pad = p->R - 1 - p->pad; a.flip = 1;
        } else {
            strided = true; a.stride = p->stride; a.pad = p->pad; a.flip = 0;
        }
    }
    // (the class form of the strided input gradient keeps at most 16 classes: larger strides take the 4-byte path)
    const bool aligned = (a.Cs % 16) == 0 && !(strided && a.stride > 4);
    if (sr_seed && out32) return HQ_E_BADARG;
    const int mode = out32 ? 0 : sr_seed ? 2 : 1;
    if (sr_seed) { a.sr.k0 = (unsigned)*sr_seed; a.sr.k1 = (unsigned)(*sr_seed >> 32); } else { a.sr.k0 = a.sr.k1 = 0; }
    a.kcols = a.taps * a.Cs;
    a.cpt = aligned ? a.Cs / 16 : 1;
    a.nchunks = aligned ? a.taps * a.cpt : (a.kcols + 15) / 16;
    // (the 4-byte path divides reduction offsets by the channel count with hq_magic_div)
    if (!aligned && (unsigned long long)a.kcols * (unsigned long long)a.Cs >= (1ull << 32)) return HQ_E_BADSHAPE;
    a.magic_Cs = hq_magic32((unsigned)a.Cs);
    a.magic_S = hq_magic32((unsigned)a.S);
    if (a.N > 64) {
        // 128-byte stages halve the barriers per tile; with enough tiles to keep three or more
        // workgroups on every compute unit, 64-byte stages (half the LDS, four resident workgroups)
        // hide more latency instead
        const long tiles = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
        // not even one 128 x 128 tile per compute unit (small images or batches under a long reduction,
        // fully connected layers): 64 x 64 tiles, four times as many workgroups
        if (aligned && !strided && mode != 2 && a.nchunks >= 16 && tiles < 256)
            return launch2m<64, 64, 2, 2, 128, false, true>(a, mode, stream);
        if (mode != 2 && a.nchunks >= 16 && !(aligned && tiles >= 3 * 256)) return launch2<128, 128, 2, 2, 128>(a, strided, aligned, mode, stream);
        return launch2<128, 128, 2, 2, 64>(a, strided, aligned, mode, stream);
    }
    if (a.N > 32 || mode == 2) return launch2<256, 64, 4, 1, 64>(a, strided, aligned, mode, stream);
    return launch2<256, 32, 4, 1, 64>(a, strided, aligned, mode, stream);
}
