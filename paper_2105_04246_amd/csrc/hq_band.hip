// Weights-resident implicit-GEMM convolution for gfx950: the fast path of hq_gemm_fwd /
// hq_gemm_dgrad (and of pass 1 of the dynamic baseline) for layers whose quantized weights fit
// in LDS next to two input patches (paper Sec. 3.1 forward / backward linear op; Sec. 3.2 and
// Sec. 4 for what the epilogue does).
//
// Mapping to the machine
//   * One workgroup of 8 wavefronts per CU owns a band of output rows of one image and walks
//     it in tiles of 256 consecutive output pixels.  The layer's weights are copied to LDS once
//     per workgroup.
//   * The 8 wavefronts form two groups of 4 (one wavefront of each group per SIMD) that work
//     half a step apart: while one group feeds the matrix cores with its tile, the other runs
//     the vector-ALU epilogue of the tile it multiplied in the previous half step.  A
//     workgroup barrier closes every half step, so MFMA and epilogue phases of the two groups
//     stay interleaved instead of colliding on the same pipe.
//   * Each group has its own input patch in LDS: the input rows its tile touches (padding ring
//     filled with the zero-point code), staged once, as they lie in memory.  im2col never
//     exists: a lane forms the address of "its" pixel under tap (r,s) when it reads the MFMA
//     fragment, so an input byte crosses L2->LDS once per tile, not once per tap.  The next
//     patch of a group is requested during its MFMA phase (into registers, a few rows between
//     taps) and written to LDS at the start of its epilogue phase, when nobody reads that patch.
//     A loader thread owns PJ 16-byte chunks of a patch row: one for rows of up to 64 pixels at 64
//     channels, two for rows of up to 126 pixels, three for the 192-channel 1x1 layers.
//   * A band whose last tile is one wavefront's worth of pixels does not spend half steps on it:
//     the second group, idle in half step 0, multiplies and requantizes it there from a third
//     patch buffer.
//   * v_mfma_i32_32x32x32_i8 with the weights as first operand: a lane then holds one output
//     pixel and, because weight rows sit in LDS in permuted order, 16 CONSECUTIVE output
//     channels, so the epilogue stores 16 codes (or 16 accumulators) per lane at once.
//   * The accumulators start from -z_a * bsum[n] (the first MFMA's addend, held in registers), so
//     they come out zero-point corrected.  Epilogue per accumulator: fold into min / max;
//     requantize with one fp32 multiply, round-half-even, clamp and pack (v_cvt_pk_u8_f32
//     saturates, which is the clamp on the full 8-bit grid).  Clipped values are counted
//     exactly, but only in 16-value groups whose own min / max requantize outside the grid
//     (requantization is monotone in the accumulator).
#include "hq_device.h"
#include <type_traits>
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
    int tail_patch;                // 1: the LDS holds a third patch, for a short last tile taken early
    int rows_per_band, bands_per_image;
    unsigned magic_Wo;             // ceil(2^32 / Wo)
    unsigned long long count;      // outputs of the whole tensor
    HqSr sr;                       // seed of stochastic rounding (epilogue mode 2)
    int sr_on;
};

constexpr int BM = 256;            // output pixels per tile: 4 wavefronts x 2 MFMA row blocks

__device__ inline int sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

template <int C> __device__ inline int wswz(int i)
{
    return (C % 128 == 0) ? (i & 7) : (C % 64 == 0) ? ((i >> 2) & 3) : ((i >> 3) & 1);
}

// PR: patch rows prefetched per tile (>= PRmax), PJ: 16-byte column chunks per thread and row.
// NG: groups of four wavefronts in a workgroup.  NG == 2: the two groups alternate matrix-core
// phase and epilogue phase in lockstep, half a step apart.  NG == 1 (when the LDS holds two
// workgroups with their own copy of the weights): a workgroup runs its phases one after the other
// and the two workgroups of a compute unit overlap freely, without a common barrier and without the
// idle half steps at both ends.
// MODE: 0 = 32-bit outputs (first pass of the dynamic baseline), 1 = fused requantization with
// round-half-even, 2 = fused with stochastic rounding (input gradients).
template <int C, int KSZ, int NT, int PR, int PJ, int NG, int MODE>
__global__ __launch_bounds__(256 * NG, NG == 1 ? 2 : 1) void hq_band_kernel(const BandArgs a)
{
    constexpr bool FUSED = MODE != 0, SR = MODE == 2;
    constexpr int BAND_THREADS = 256 * NG;
    constexpr int NCH = C / 16, KS = C / 32, PP = C + 16, BN = 32 * NT, TAPS = KSZ * KSZ;
    constexpr int WROW = TAPS * C;                        // bytes per weight row in LDS
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    const int patch_bytes = a.PRmax * a.PW * PP;
    int8_t *Wl = smem;                                     // [npad][TAPS][C], chunks swizzled
    int *bz = reinterpret_cast<int *>(smem + (size_t)a.npad * WROW);     // [npad]  z_a * bsum[n]
    int8_t *Pl = reinterpret_cast<int8_t *>(bz + a.npad);  // one patch per group [PRmax * PW][PP]
    int8_t *Pt = Pl + NG * (size_t)patch_bytes;            // patch of an early last tile (if a.tail_patch)
    int *red = reinterpret_cast<int *>(Pl + (NG + a.tail_patch) * (size_t)patch_bytes);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: branches on it are uniform
    const int grp = NG == 2 ? wave >> 2 : 0, gwave = wave & 3, gtid = tid & 255;
    int8_t *Pg = Pl + grp * patch_bytes;                   // this group's patch

    // ---- start-up, part 1: everything that does not depend on other loads is requested before anything
    // waits (the first pass of the weight copy, the weight sums, then the scalars below), so that the
    // memory round trips of the start-up overlap instead of following one another.
    // Every workgroup copies the same weights: each starts at another place of the array, so that
    // the workgroups of a launch do not walk the same cache lines in the same order.
    constexpr int WB = 6;
    const int wchunks = a.npad * TAPS * NCH;
    const int wrot = (int)(((blockIdx.x & 15u) * (unsigned)wchunks) >> 4) & ~7;
    auto rotated = [&](int i) { const int r = i + wrot; return r >= wchunks ? r - wchunks : r; };
    auto wload = [&](int base, v4i (&wv)[WB]) {
#pragma unroll
        for (int k = 0; k < WB; k++) {
            const int lin = base + tid + BAND_THREADS * k, idx = rotated(lin);
            const int cq = idx % NCH, t = (idx / NCH) % TAPS, row = idx / (NCH * TAPS);
            const int n = (row & ~31) + sigma32(row & 31);
            const int tsrc = a.flip ? TAPS - 1 - t : t;
            wv[k] = v4i{0, 0, 0, 0};
            if (lin < wchunks && n < a.N)
                wv[k] = *reinterpret_cast<const v4i *>(a.Bw + ((size_t)n * TAPS + tsrc) * C + cq * 16);
        }
    };
    auto wstore = [&](int base, const v4i (&wv)[WB]) {
#pragma unroll
        for (int k = 0; k < WB; k++) {
            const int lin = base + tid + BAND_THREADS * k, idx = rotated(lin);
            const int cq = idx % NCH, t = (idx / NCH) % TAPS, row = idx / (NCH * TAPS);
            if (lin < wchunks)
                *reinterpret_cast<v4i *>(Wl + row * WROW + t * C + 16 * (cq ^ wswz<C>(row & 31))) = wv[k];
        }
    };
    v4i wv0[WB];
    wload(0, wv0);
    const int bs0 = tid < a.N ? a.bsum[tid] : 0;
    const int za = a.aq->zero_point;
    const int fillw = (int)((unsigned)(za & 0xff) * 0x01010101u);   // unsigned: the product may set bit 31
    const v4i fill = {fillw, fillw, fillw, fillw};

    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);

    // ---- this workgroup's band
    const int img = blockIdx.x / a.bands_per_image, band = blockIdx.x % a.bands_per_image;
    const int row0 = band * a.rows_per_band, row1 = min(a.Ho, row0 + a.rows_per_band);
    const int p0 = row0 * a.Wo, p1 = row1 * a.Wo;
    const int ntile = (p1 - p0 + BM - 1) / BM;
    const int nchunk = a.npad / BN;
    const int nitem = ntile * nchunk;                      // work items: (tile, column chunk)
    const int8_t *Aimg = a.A + (size_t)img * a.Hs * a.Ws * C;
    const size_t out_img = (size_t)img * a.Ho * a.Wo;

    // ---- patch loader: thread <-> fixed column chunk(s) of a patch row; slot <-> patch row
    int col_src[PJ], col_lds[PJ];
    bool col_ok[PJ], col_in[PJ];
#pragma unroll
    for (int j = 0; j < PJ; j++) {
        const int cidx = gtid + 256 * j, ixp = cidx / NCH, q = cidx % NCH, ix = ixp - a.pad;
        col_in[j] = cidx < a.PW * NCH;                     // inside the patch row at all
        col_ok[j] = col_in[j] && ix >= 0 && ix < a.Ws;     // ... and inside the image
        col_src[j] = ix * C + q * 16;
        col_lds[j] = ixp * PP + q * 16;
    }
    v4i pf[PR][PJ];
    int pf_nrows = 0, pf_iy = 0;                           // rows of the patch being prefetched, its first input row
    auto prefetch_setup = [&](int tile) {
        const int ps = p0 + tile * BM;
        const int oy0 = (int)hq_magic_div((unsigned)ps, a.magic_Wo);
        const int oy1 = (int)hq_magic_div((unsigned)(min(ps + BM, p1) - 1), a.magic_Wo);
        pf_nrows = (oy1 - oy0) * a.stride + KSZ;
        pf_iy = oy0 * a.stride - a.pad;
    };
    auto prefetch_row = [&](int k) {                       // k < PR, compile-time at every call site
        const int iy = pf_iy + k;
        const bool row_ok = k < pf_nrows && iy >= 0 && iy < a.Hs;        // uniform
        const int8_t *rowp = Aimg + (size_t)(row_ok ? iy : 0) * a.Ws * C;
#pragma unroll
        for (int j = 0; j < PJ; j++) {
            v4i v = fill;
            if (row_ok && col_ok[j]) v = *reinterpret_cast<const v4i *>(rowp + col_src[j]);
            pf[k][j] = v;
        }
    };
    auto prefetch = [&](int tile) {
        prefetch_setup(tile);
#pragma unroll
        for (int k = 0; k < PR; k++) prefetch_row(k);
    };
    auto stash = [&](int8_t *dst) {
#pragma unroll
        for (int k = 0; k < PR; k++)
#pragma unroll
            for (int j = 0; j < PJ; j++)
                if (k < a.PRmax && col_in[j])
                    *reinterpret_cast<v4i *>(dst + k * a.PW * PP + col_lds[j]) = pf[k][j];
    };

    // ---- start-up: request the group's first patch and the weights before anything waits
    // A last tile that one wavefront covers does not get half steps of its own: the second group,
    // which would idle through half step 0, multiplies and requantizes it there, from a patch
    // buffer of its own (so that the group's first regular patch can be written meanwhile).
    const bool early_tail = NG == 2 && a.tail_patch && nchunk == 1 && nitem >= 2 && (p1 - p0) - (ntile - 1) * BM <= 64;
    const int nmain = early_tail ? nitem - 1 : nitem;      // items that take turns in the half steps
    const bool tail_grp = early_tail && grp == 1;
    if (tail_grp) {
        prefetch(ntile - 1);
        stash(Pt);
    }
    if (grp < nmain) prefetch(grp / nchunk);
    wstore(0, wv0);
    for (int base = BAND_THREADS * WB; base < wchunks; base += BAND_THREADS * WB) {
        v4i wv[WB];
        wload(base, wv);
        wstore(base, wv);
    }
    if (tid < a.npad) bz[tid] = za * bs0;
    for (int n = tid + BAND_THREADS; n < a.npad; n += BAND_THREADS) bz[n] = n < a.N ? za * a.bsum[n] : 0;
    if (grp < nmain && !tail_grp) stash(Pg);               // the tail group keeps its first patch in registers
    __syncthreads();

    // per-lane weight fragment addresses (row i = lane % 32 of each 32-row block)
    int wbase[NT][KS];
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            wbase[j][ks] = (j * 32 + (lane & 31)) * WROW + 16 * ((ks * 2 + (lane >> 5)) ^ wswz<C>(lane & 31));

    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;
    v16i acc[2][NT];
    int pix[2] = {0, 0};
    bool ok[2] = {false, false};
    bool have_pf = false;

    // -z_a * bsum[n] of the lane's 16 channels per column block: the matrix cores' first addend
    v16i nbz[NT];
    int nbz_chunk = -1;

    // Half step h: item h is multiplied (by group h & 1) while item h-1 goes through the
    // epilogue (in the other group, which multiplied it during half step h-1).
    const int nhalf = NG == 2 ? nmain + 1 : 2 * nitem;
    for (int h = 0; h < nhalf; h++) {
      const bool tail_now = tail_grp && h == 0;
      const int8_t *Psrc = tail_now ? Pt : Pg;
      for (int sub = 0; sub < (tail_now ? 2 : 1); sub++) {
        const bool mfma_phase = tail_now ? sub == 0 : NG == 2 ? (h & 1) == grp : (h & 1) == 0;
        // this group's item in this half step
        const int item = tail_now ? nitem - 1 : NG == 2 ? (mfma_phase ? h : h - 1) : h >> 1;
        if (item >= 0 && (item < nmain || tail_now)) {
            const int tile = nchunk == 1 ? item : item / nchunk, nc = item - tile * nchunk;
            const int ps = p0 + tile * BM;
            if (mfma_phase) {
                // -------------------------------------------------- matrix-core phase
                if (tail_now && grp < nmain) stash(Pg);    // nobody reads this group's patch in this half step
                const int nxt = item + NG;
                have_pf = !tail_now && nxt < nmain && (nchunk == 1 || nxt / nchunk != tile);
                const bool active = ps + gwave * 64 < p1;
                // the next tile's patch rows are requested between the taps (a few per tap), where the
                // wait for a slot in the memory pipeline overlaps the MFMAs already issued
                constexpr int RPT = (PR + TAPS - 1) / TAPS;
                if (have_pf) {
                    prefetch_setup(nchunk == 1 ? nxt : nxt / nchunk);
                    if (!active) {
#pragma unroll
                        for (int k = 0; k < PR; k++) prefetch_row(k);
                    }
                }
                const int oy0 = (int)hq_magic_div((unsigned)ps, a.magic_Wo);
                int abase[2];
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    const int p = ps + gwave * 64 + i * 32 + (lane & 31);
                    ok[i] = p < p1;
                    pix[i] = ok[i] ? p : ps;
                    const int oy = (int)hq_magic_div((unsigned)pix[i], a.magic_Wo), ox = pix[i] - oy * a.Wo;
                    abase[i] = (((oy - oy0) * a.stride) * a.PW + ox * a.stride) * PP + (lane >> 5) * 16;
                }
                if (nc != nbz_chunk) {
                    nbz_chunk = nc;
#pragma unroll
                    for (int j = 0; j < NT; j++)
#pragma unroll
                        for (int g = 0; g < 4; g++) {
                            const v4i bzv = *reinterpret_cast<const v4i *>(bz + nc * BN + j * 32 + 16 * (lane >> 5) + 4 * g);   // < npad
#pragma unroll
                            for (int e = 0; e < 4; e++) nbz[j][4 * g + e] = -bzv[e];
                        }
                }
                if (active) {
                    // Fragments of tap t+1 are requested before the MFMAs of tap t are issued, so
                    // LDS latency hides behind the matrix cores (two register buffers).
                    const int8_t *Wc = Wl + nc * BN * WROW;
                    v4i wfA[KS][NT], afA[KS][2], wfB[KS][NT], afB[KS][2];
                    auto load_tap = [&](int t, v4i (&wf)[KS][NT], v4i (&af)[KS][2]) {
                        const int toff = ((t / KSZ) * a.PW + (t % KSZ)) * PP;
#pragma unroll
                        for (int ks = 0; ks < KS; ks++) {
#pragma unroll
                            for (int j = 0; j < NT; j++)
                                wf[ks][j] = *reinterpret_cast<const v4i *>(Wc + wbase[j][ks] + t * C);
#pragma unroll
                            for (int i = 0; i < 2; i++)
                                af[ks][i] = *reinterpret_cast<const v4i *>(Psrc + abase[i] + toff + ks * 32);
                        }
                    };
                    auto mfma_tap = [&](v4i (&wf)[KS][NT], v4i (&af)[KS][2], auto first) {
#pragma unroll
                        for (int ks = 0; ks < KS; ks++)
#pragma unroll
                            for (int i = 0; i < 2; i++)
#pragma unroll
                                for (int j = 0; j < NT; j++)
                                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                        wf[ks][j], af[ks][i], (decltype(first)::value && ks == 0) ? nbz[j] : acc[i][j], 0, 0, 0);
                    };
                    // the fragment reads of tap t + 1 are dealt between the MFMAs of tap t (a wavefront issues in
                    // order; an MFMA holds the matrix pipe for 32 cycles in which seven other instructions can go)
                    auto interleave = [&]() {
#pragma unroll
                        for (int q = 0; q < KS * (NT + 2); q++) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
                            __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);     // one vector ALU instruction
                        }
                        __builtin_amdgcn_sched_group_barrier(0x008, KS * 2 * NT, 0);
                    };
                    load_tap(0, wfA, afA);
#pragma unroll
                    for (int t = 0; t < TAPS; t += 2) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (t + 1 < TAPS) load_tap(t + 1, wfB, afB);
                        if (t == 0) mfma_tap(wfA, afA, std::true_type()); else mfma_tap(wfA, afA, std::false_type());
                        if (t + 1 < TAPS) interleave();
                        __builtin_amdgcn_sched_barrier(0);
                        if (have_pf) {
#pragma unroll
                            for (int k = t * RPT; k < (t + 1) * RPT && k < PR; k++) prefetch_row(k);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (t + 2 < TAPS) load_tap(t + 2, wfA, afA);
                        if (t + 1 < TAPS) {
                            mfma_tap(wfB, afB, std::false_type());
                            if (t + 2 < TAPS) interleave();
                            __builtin_amdgcn_sched_barrier(0);
                            if (have_pf) {
#pragma unroll
                                for (int k = (t + 1) * RPT; k < (t + 2) * RPT && k < PR; k++) prefetch_row(k);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
                // -------------------------------------------------- vector-ALU phase
                if (have_pf) stash(Pg);                    // nobody reads this group's patch now
                auto epilogue = [&](auto full) {
                    constexpr bool FULL = decltype(full)::value;
#pragma unroll
                    for (int i = 0; i < 2; i++) {
                        if (!ok[i]) continue;
                        const size_t m = out_img + pix[i];
#pragma unroll
                        for (int j = 0; j < NT; j++) {
                            const int nb = nc * BN + j * 32 + 16 * (lane >> 5);
                            if (nb >= a.N) continue;
                            int c[16];
#pragma unroll
                            for (int r = 0; r < 16; r++) c[r] = acc[i][j][r];
                            if (FUSED) {
                                int w[4];
                                if (SR) hq_requant_group_sr<16, FULL>(c, ep, a.sr, m * a.N + nb, mn, mx, nlo, nhi, w);
                                else hq_requant_group<16, FULL>(c, ep, mn, mx, nlo, nhi, w);
                                const v4i packed = {w[0], w[1], w[2], w[3]};
                                *reinterpret_cast<v4i *>(a.out8 + m * a.N + nb) = packed;
                            } else {
                                hq_minmax_group<16>(c, mn, mx);
#pragma unroll
                                for (int g = 0; g < 4; g++) {
                                    const v4i v = {c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                                    *reinterpret_cast<v4i *>(a.out32 + m * a.N + nb + 4 * g) = v;
                                }
                            }
                        }
                    }
                };
                if (ep.full_grid) epilogue(std::true_type()); else epilogue(std::false_type());
            }
        }
      }
        __syncthreads();
    }

    hq_block_stats_commit_n<BAND_THREADS>(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, a.count);
        if (FUSED) *a.outq = a.range->qp;
    }
}

constexpr size_t BAND_LDS_MAX = 160 * 1024;

template <int C, int KSZ, int NT, int PR, int PJ, int NG, int MODE>
int launch_band_mode(const BandArgs &a, int blocks, size_t lds, hipStream_t s)
{
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(hq_band_kernel<C, KSZ, NT, PR, PJ, NG, MODE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)BAND_LDS_MAX) != hipSuccess)
            return HQ_E_HIP;
        configured = true;
    }
    hipLaunchKernelGGL((hq_band_kernel<C, KSZ, NT, PR, PJ, NG, MODE>), dim3(blocks), dim3(256 * NG), lds, s, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

template <int C, int KSZ, int NT, int PR, int PJ, int NG>
int launch_band(const BandArgs &a, int mode, int blocks, size_t lds, hipStream_t s)
{
    if (mode == 0) return launch_band_mode<C, KSZ, NT, PR, PJ, NG, 0>(a, blocks, lds, s);
    if (mode == 1) return launch_band_mode<C, KSZ, NT, PR, PJ, NG, 1>(a, blocks, lds, s);
    return launch_band_mode<C, KSZ, NT, PR, PJ, NG, 2>(a, blocks, lds, s);
}

template <int C, int KSZ, int NT, int PR, int PJ>
int launch_band_ng(const BandArgs &a, int ng, int blocks, size_t lds, hipStream_t s)
{
    const int mode = a.out32 ? 0 : a.sr_on ? 2 : 1;
    return ng == 1 ? launch_band<C, KSZ, NT, PR, PJ, 1>(a, mode, blocks, lds, s)
                   : launch_band<C, KSZ, NT, PR, PJ, 2>(a, mode, blocks, lds, s);
}

} // namespace

// Returns HQ_OK after launching, HQ_E_BADSHAPE if this path does not cover the problem (the
// caller then uses the general gather kernel), HQ_E_HIP on a launch error.
int hq_try_launch_band(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                       const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                       int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed)
{
    if (p->kind != HQ_CONV2D || p->R != p->S) return HQ_E_BADSHAPE;
    if (dgrad && p->stride != 1) return HQ_E_BADSHAPE;
    if (sr_seed && out32) return HQ_E_BADARG;
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    BandArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.sr_on = sr_seed != nullptr;
    a.sr = sr_seed ? HqSr{(unsigned)*sr_seed, (unsigned)(*sr_seed >> 32)} : HqSr{0, 0};
    int C;
    if (!dgrad) {
        C = p->C; a.N = p->Cout; a.Hs = p->H; a.Ws = p->W; a.Ho = OH; a.Wo = OW;
        a.stride = p->stride; a.pad = p->pad; a.flip = 0;
    } else {
        C = p->Cout; a.N = p->C; a.Hs = OH; a.Ws = OW; a.Ho = p->H; a.Wo = p->W;
        a.stride = 1; a.pad = p->R - 1 - p->pad; a.flip = 1;
    }
    const int KSZ = p->R;
    int NT, PJ;
    if (C == 64 && KSZ == 3) { NT = 2; PJ = ((a.Wo - 1) * a.stride + KSZ) * 4 > 256 ? 2 : 1; }   // patch rows of up to 64 / 128 pixels
    else if (C == 32 && KSZ == 1) { NT = 2; PJ = 1; }
    else if (C == 192 && KSZ == 1) { NT = 1; PJ = 3; }
    else return HQ_E_BADSHAPE;
    if ((a.N % 16) != 0 || a.Ho * a.Wo >= 65536) return HQ_E_BADSHAPE;
    const int BN = 32 * NT;
    a.npad = (a.N + BN - 1) / BN * BN;
    a.PW = (a.Wo - 1) * a.stride + KSZ;
    if (a.PW * (C / 16) > 256 * PJ) return HQ_E_BADSHAPE;

    // bands: one two-group workgroup per CU, or (1x1 layers, where it measured faster: short tiles,
    // small weights) two independent one-group workgroups when the LDS holds both
    size_t lds = 0;
    int ng = 1, prmax = 0;
    for (ng = KSZ == 1 ? 1 : 2; ng <= 2; ng++) {
        int bpi = ((ng == 1 ? 512 : 256) + p->B - 1) / p->B;
        if (bpi > a.Ho) bpi = a.Ho;
        if (bpi < 1) bpi = 1;
        a.rows_per_band = (a.Ho + bpi - 1) / bpi;
        a.bands_per_image = (a.Ho + a.rows_per_band - 1) / a.rows_per_band;
        // most patch rows any tile needs
        prmax = 0;
        for (int band = 0; band < a.bands_per_image; band++) {
            const int r0 = band * a.rows_per_band, r1 = (r0 + a.rows_per_band < a.Ho) ? r0 + a.rows_per_band : a.Ho;
            for (int ps = r0 * a.Wo; ps < r1 * a.Wo; ps += BM) {
                const int last = (ps + BM < r1 * a.Wo ? ps + BM : r1 * a.Wo) - 1;
                const int rows = (last / a.Wo - ps / a.Wo) * a.stride + KSZ;
                if (rows > prmax) prmax = rows;
            }
        }
        lds = (size_t)a.npad * KSZ * KSZ * C + (size_t)a.npad * 4 + ng * (size_t)prmax * a.PW * (C + 16) + 128;
        if (ng == 1 && 2 * (lds + 1024) <= BAND_LDS_MAX) break;      // two workgroups fit (1 KiB each of slack)
        if (ng == 2) break;
    }
    a.PRmax = prmax;
    a.tail_patch = 0;
    if (ng == 2 && lds + (size_t)prmax * a.PW * (C + 16) <= BAND_LDS_MAX) {
        a.tail_patch = 1;
        lds += (size_t)prmax * a.PW * (C + 16);
    }
    if (lds > BAND_LDS_MAX) return HQ_E_BADSHAPE;
    a.magic_Wo = hq_magic32((unsigned)a.Wo);
    a.count = (unsigned long long)p->B * a.Ho * a.Wo * a.N;
    const int blocks = p->B * a.bands_per_image;
    if (C == 64 && PJ == 2) {
        if (prmax <= 6) return launch_band_ng<64, 3, 2, 6, 2>(a, ng, blocks, lds, stream);
        return HQ_E_BADSHAPE;
    }
    if (C == 64) {
        if (prmax <= 8) return launch_band_ng<64, 3, 2, 8, 1>(a, ng, blocks, lds, stream);
        if (prmax <= 12) return launch_band_ng<64, 3, 2, 12, 1>(a, ng, blocks, lds, stream);
        return HQ_E_BADSHAPE;
    }
    if (C == 32) {
        if (prmax <= 6) return launch_band_ng<32, 1, 2, 6, 1>(a, ng, blocks, lds, stream);
        if (prmax <= 14) return launch_band_ng<32, 1, 2, 14, 1>(a, ng, blocks, lds, stream);
        return HQ_E_BADSHAPE;
    }
    if (prmax <= 6) return launch_band_ng<192, 1, 1, 6, 3>(a, ng, blocks, lds, stream);
    return HQ_E_BADSHAPE;
}
