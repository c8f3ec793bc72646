// 3x3 stride-1 convolution with 128 or more channels on int8 MFMA with the fused in-hindsight epilogue:
// forward and, with mirrored taps, the input gradient of the layers of ResNet stages 2 to 4 and of
// VGG's later blocks (paper Sec. 3.1; Sec. 3.2 static quantization; Sec. 4 steps 1 and 2).
//
// Tiling.  The output is a matrix of M = B * H * W pixels (flat NHWC order) by N channels.  A workgroup of
// four wavefronts (one per SIMD, one workgroup per compute unit) owns a tile of TM consecutive pixels by
// TN channels; the wavefronts form a 2 x 2 grid and each holds MT x NT MFMA blocks of 32 x 32
// (up to 128 pixels x 128 channels: 256 accumulators per lane, which live in the accumulation registers).
// Large wavefront tiles are what the matrix cores need here: a 32 x 32 x 32 MFMA takes 32 cycles and a
// fragment read from LDS 8, so a wavefront tile of a x b blocks reads (a + b) fragments per a * b MFMAs.
// Tiles are cut from the flat pixel index, not from image rows, so that images of 14 x 14 or 7 x 7 pixels
// fill the MFMA blocks as well as large ones.
//
// Data movement.  The input pixels of a tile are staged once per 64-channel chunk together with their
// one-pixel border (the zero-point code outside the image): the patch holds every input row the tile's
// output rows touch, each image with its own border rows, and the nine taps are nine shifted views of it.
// The weights stream through LDS in steps of one (tap, 64-channel chunk): TN rows of 64 bytes, two steps
// per stage, three stages in LDS: the loads of stage s + 2 are requested when stage s begins, and the
// wait that closes stage s only asks for stage s + 1 (requested a whole stage earlier), because a load that
// every compute unit issues at the same moment takes longer than one stage's MFMAs.  Everything goes
// global -> LDS without passing through registers (global_load_lds_dwordx4: lane l of a wavefront lands at
// base + 16 * l), so LDS rows are dense and their four 16-byte chunks are XOR-swizzled by the row index,
// applied to the chunk a lane fetches.
//
// The reduction loop has no branch between its LDS reads and its MFMAs: the fragments of k-step k + 1 are
// requested before the MFMAs of k-step k are issued, and the counter waits the compiler derives for
// straight-line code let the reads of one k-step complete under the MFMAs of the other.
#include "hq_device.h"
#include "hq_internal.h"
#include <type_traits>

namespace {

constexpr int C3_CK = 64;          // channels per reduction chunk (bytes per LDS row)
constexpr size_t C3_LDS_MAX = 160 * 1024;

struct Conv3Args {
    const int8_t *A, *Bw;
    const int32_t *bsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int Bn, H, W, C, N;            // stride 1, pad 1: the output image is H x W
    int flip;                      // weight taps mirrored (dgrad)
    int M;                         // Bn * H * W
    int ntiles, nchunks;           // pixel tiles, TN-channel chunks of the output
    int PW, H2;                    // patch row length (W + 2), padded rows per image (H + 2)
    int patch_bytes;               // one patch buffer, a multiple of 1024
    unsigned magic_W, magic_H, magic_PW, magic_H2;
    unsigned long long count;
    HqSr sr;                       // seed of stochastic rounding (epilogue mode 2)
};

__device__ inline int c3_sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }
__device__ inline int c3_swz(int row) { return (row >> 2) & 3; }

// MT x NT: MFMA blocks per wavefront (tile = 64 MT pixels x 64 NT channels).
// MODE: 0 = 32-bit outputs, 1 = fused requantization with round-half-even, 2 = fused with stochastic rounding.
template <int MT, int NT, int MODE>
__global__ __launch_bounds__(HQ_THREADS, 1) void hq_conv3_kernel(const Conv3Args a)
{
    constexpr bool FUSED = MODE != 0, SR = MODE == 2;
    constexpr int TM = 64 * MT, TN = 64 * NT;
    constexpr int WSTEP = TN * C3_CK;                      // bytes of one weight step in LDS
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t *Wl = smem;                                     // [3 stages][2 steps][TN][64]
    int8_t *Pl = smem + 6 * WSTEP;                         // [2][patch_bytes]
    int *bz = reinterpret_cast<int *>(Pl + 2 * (size_t)a.patch_bytes);     // [TN]
    int *red = bz + TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int za = a.aq->zero_point;
    const int fillw = (int)((unsigned)(za & 0xff) * 0x01010101u);
    const v4i fillv = {fillw, fillw, fillw, fillw};
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);
    const int cchunks = a.C / C3_CK, nsteps = cchunks * 9, nfull = nsteps >> 1;
    const size_t wrow = (size_t)9 * a.C;                   // bytes of a weight row

    // weight fragment offsets inside a step (row block j adds j * 32 * 64; the swizzle repeats every 8 rows)
    int wfoff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ks++)
        wfoff[ks] = (wn * NT * 32 + (lane & 31)) * C3_CK + 16 * ((2 * ks + half) ^ c3_swz(lane & 31));

    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;

    for (int item = blockIdx.x; item < a.ntiles * a.nchunks; item += gridDim.x) {
        const int tile = item / a.nchunks, nc = item - tile * a.nchunks;
        const int n0 = nc * TN, m0 = tile * TM;
        // ---- the patch: padded input rows pr0 .. pr0 + nrows - 1, padded row of (image b, input row iy) = b * H2 + iy + 1
        const int g0 = (int)hq_magic_div((unsigned)m0, a.magic_W);
        const int g1 = (int)hq_magic_div((unsigned)(min(m0 + TM, a.M) - 1), a.magic_W);
        const int b0 = (int)hq_magic_div((unsigned)g0, a.magic_H), b1 = (int)hq_magic_div((unsigned)g1, a.magic_H);
        const int pr0 = b0 * a.H2 + (g0 - b0 * a.H);                       // input row y - 1 of the first output row
        const int nrows = b1 * a.H2 + (g1 - b1 * a.H) + 2 - pr0 + 1;       // ... up to input row y + 1 of the last one
        const int patch_slots = nrows * a.PW * 4;                          // 16-byte chunks

        __syncthreads();                                   // the previous item's readers are done with bz and LDS
        if (tid < TN) bz[tid] = n0 + tid < a.N ? za * a.bsum[n0 + tid] : 0;

        // ---- loaders.  Patch chunk: LDS slot q -> patch pixel q / 4, 16-byte chunk q % 4 (swizzled source).
        auto issue_patch = [&](int cchunk, int buf) {
            int8_t *dstp = Pl + (size_t)buf * a.patch_bytes;
            for (int q0 = 0; q0 < patch_slots; q0 += HQ_THREADS) {
                const int q = q0 + tid;
                const int ppix = q >> 2, ck = (q & 3) ^ c3_swz(ppix);
                const int prow = (int)hq_magic_div((unsigned)ppix, a.magic_PW), pc = ppix - prow * a.PW;
                const int pr = pr0 + prow;
                const int b = (int)hq_magic_div((unsigned)pr, a.magic_H2), iy = pr - b * a.H2 - 1, ix = pc - 1;
                const bool inside = q < patch_slots && b < a.Bn && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                int8_t *dst = dstp + (size_t)(q0 + (tid & ~63)) * 16;   // this wavefront's 1 KiB
                if (inside) {
                    const int8_t *src = a.A + (((size_t)b * a.H + iy) * a.W + ix) * a.C + cchunk * C3_CK + ck * 16;
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                     (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
                } else if (q < ((patch_slots + 63) & ~63)) {
                    *reinterpret_cast<v4i *>(dst + lane * 16) = fillv;
                }
            }
        };
        // Weight step: LDS row = channel sigma-permuted inside its 32-block, slot q -> row q / 4, chunk q % 4.
        // Rows past the last channel repeat the last one: their outputs are never stored, and every lane
        // issues the same number of loads, which the counter wait at the end of a stage relies on.
        const int8_t *wsrc[NT];
#pragma unroll
        for (int k = 0; k < NT; k++) {
            const int q = tid + HQ_THREADS * k, row = q >> 2, ck = (q & 3) ^ c3_swz(row);
            const int n = min(n0 + (row & ~31) + c3_sigma32(row & 31), a.N - 1);
            wsrc[k] = a.Bw + (size_t)n * wrow + ck * 16;
        }
        auto issue_step = [&](int step, int slot) {           // slot = stage buffer * 2 + step inside the stage
            const int cchunk = step / 9, tap = step - cchunk * 9;
            const int woff = (a.flip ? 8 - tap : tap) * a.C + cchunk * C3_CK;
#pragma unroll
            for (int k = 0; k < NT; k++) {
                int8_t *dst = Wl + (size_t)slot * WSTEP + (size_t)(HQ_THREADS * k + (tid & ~63)) * 16;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wsrc[k] + woff),
                                                 (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
            }
        };
        auto issue_stage = [&](int stage) {
            const int slot = (stage % 3) * 2;
            issue_step(2 * stage, slot);
            if (2 * stage + 1 < nsteps) issue_step(2 * stage + 1, slot + 1);
        };

        issue_patch(0, 0);
        issue_stage(0);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        if (nsteps > 2) issue_stage(1);                     // in flight while the first stage is multiplied

        // ---- this lane's pixels: patch pixel of tap (0, 0), and whether they exist
        int ppx[MT];
        bool ok[MT];
#pragma unroll
        for (int i = 0; i < MT; i++) {
            const int m = m0 + wm * (32 * MT) + i * 32 + (lane & 31);
            ok[i] = m < a.M;
            const int mm = ok[i] ? m : m0;
            const int g = (int)hq_magic_div((unsigned)mm, a.magic_W), x = mm - g * a.W;
            const int b = (int)hq_magic_div((unsigned)g, a.magic_H), y = g - b * a.H;
            ppx[i] = (b * a.H2 + y - pr0) * a.PW + x;
        }

        __syncthreads();

        v16i acc[MT][NT];
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const v4i bzv = *reinterpret_cast<const v4i *>(bz + (wn * NT + j) * 32 + 16 * half + 4 * g);
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[i][j][4 * g + e] = -bzv[e];
            }

        // fragments of one k-step: NT weight blocks, MT pixel blocks
        auto load_frags = [&](const int8_t *Wb, const int8_t *Pb, int toff, int ks, v4i (&wf)[NT], v4i (&af)[MT]) {
#pragma unroll
            for (int j = 0; j < NT; j++) wf[j] = *reinterpret_cast<const v4i *>(Wb + j * 32 * C3_CK + wfoff[ks]);
#pragma unroll
            for (int i = 0; i < MT; i++) {
                const int row = ppx[i] + toff;
                af[i] = *reinterpret_cast<const v4i *>(Pb + row * C3_CK + 16 * ((2 * ks + half) ^ c3_swz(row)));
            }
        };
        auto mfmas = [&](const v4i (&wf)[NT], const v4i (&af)[MT]) {
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], acc[i][j], 0, 0, 0);
        };
        auto step_place = [&](int step, const int8_t *&Pb, int &toff) {
            const int cchunk = step / 9, tap = step - cchunk * 9;
            Pb = Pl + (size_t)(cchunk & 1) * a.patch_bytes;
            toff = (tap / 3) * a.PW + (tap % 3);
        };

        v4i wfA[NT], afA[MT], wfB[NT], afB[MT];
        for (int s = 0; s < nfull; s++) {
            // requests first: the next chunk's patch (by the first stage that lies wholly inside this chunk:
            // every reader of the buffer it overwrites finished before that stage's opening barrier), then the
            // next stage's weights
            {
                const int c0 = (2 * s) / 9, t0 = 2 * s - c0 * 9;
                if (t0 <= 1 && c0 + 1 < cchunks) issue_patch(c0 + 1, (c0 + 1) & 1);
            }
            const int ahead = nsteps - 2 * (s + 2);         // steps of stage s + 2 (<= 0: none)
            if (ahead > 0) issue_stage(s + 2);
            __builtin_amdgcn_sched_barrier(0);
            // four k-steps (two per step), straight-line
            const int8_t *W0 = Wl + (size_t)((s % 3) * 2) * WSTEP, *W1 = W0 + WSTEP, *P0, *P1;
            int toff0, toff1;
            step_place(2 * s, P0, toff0);
            step_place(2 * s + 1, P1, toff1);
            load_frags(W0, P0, toff0, 0, wfA, afA);
            load_frags(W0, P0, toff0, 1, wfB, afB);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfA, afA);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(W1, P1, toff1, 0, wfA, afA);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfB, afB);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(W1, P1, toff1, 1, wfB, afB);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfA, afA);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfB, afB);
            __builtin_amdgcn_sched_barrier(0);
            // everything but the loads requested in this iteration's last batch (stage s + 2: NT loads per
            // step and lane, issued after any patch loads) has to have landed: stage s + 1 and the patch
            if (ahead >= 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * NT) : "memory");
            else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NT) : "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __syncthreads();
        }
        if (nsteps & 1) {                                   // the last, single step (its stage was requested above)
            const int8_t *W0 = Wl + (size_t)((nfull % 3) * 2) * WSTEP, *P0;
            int toff0;
            step_place(nsteps - 1, P0, toff0);
            load_frags(W0, P0, toff0, 0, wfA, afA);
            load_frags(W0, P0, toff0, 1, wfB, afB);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfA, afA);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(wfB, afB);
        }

        // ---- epilogue: lane = one pixel per 32-row block, 16 consecutive channels per column block
        auto epilogue = [&](auto full) {
            constexpr bool FULL = decltype(full)::value;
#pragma unroll
            for (int i = 0; i < MT; i++) {
                if (!ok[i]) continue;
                const size_t m = (size_t)m0 + wm * (32 * MT) + i * 32 + (lane & 31);
#pragma unroll
                for (int j = 0; j < NT; j++) {
                    const int nb = n0 + (wn * NT + j) * 32 + 16 * half;
                    if (nb >= a.N) continue;               // N % 16 == 0: a group is all in or all out
                    int c[16];
#pragma unroll
                    for (int e = 0; e < 16; e++) c[e] = acc[i][j][e];
                    const size_t o = m * a.N + nb;
                    if (FUSED) {
                        int w[4];
                        if (SR) hq_requant_group_sr<16, FULL>(c, ep, a.sr, o, mn, mx, nlo, nhi, w);
                        else hq_requant_group<16, FULL>(c, ep, mn, mx, nlo, nhi, w);
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
    }
    __syncthreads();
    hq_block_stats_commit(mn, mx, nlo, nhi, a.st, red);
    if (blockIdx.x == 0 && tid == 0) {
        a.st->acc_scale = acc_scale;
        atomicAdd((unsigned long long *)&a.st->count, a.count);
        if (FUSED) *a.outq = a.range->qp;
    }
}

// Patch rows a tile of TM flat pixels can touch: its output rows, one border row above and below, and two
// more border rows for every further image it runs into.
int c3_patch_rows(int TM, int H, int W)
{
    const int rows_out = (TM + W - 2) / W + 1;
    const int images = (rows_out + H - 2) / H + 1;
    return rows_out + 2 * images;
}

template <int MT, int NT>
size_t c3_lds_bytes(const hq_problem *p)
{
    const size_t patch = ((size_t)c3_patch_rows(64 * MT, p->H, p->W) * (p->W + 2) * C3_CK + 1023) & ~(size_t)1023;
    return 6 * (size_t)(64 * NT) * C3_CK + 2 * patch + 4 * (64 * NT) + 64;
}

template <int MT, int NT, int MODE>
int c3_launch_mode(Conv3Args &a, const hq_problem *p, hipStream_t stream)
{
    const int TM = 64 * MT, TN = 64 * NT;
    a.ntiles = (a.M + TM - 1) / TM;
    a.nchunks = (a.N + TN - 1) / TN;
    a.patch_bytes = (int)(((size_t)c3_patch_rows(TM, p->H, p->W) * (p->W + 2) * C3_CK + 1023) & ~(size_t)1023);
    const size_t lds = c3_lds_bytes<MT, NT>(p);
    auto kern = hq_conv3_kernel<MT, NT, MODE>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)C3_LDS_MAX) != hipSuccess)
            return HQ_E_HIP;
        configured = true;
    }
    const long items = (long)a.ntiles * a.nchunks;
    const int blocks = (int)(items < 256 ? items : 256);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(HQ_THREADS), lds, stream, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}

template <int MT, int NT>
int c3_launch(Conv3Args &a, const hq_problem *p, int mode, hipStream_t stream)
{
    if (mode == 0) return c3_launch_mode<MT, NT, 0>(a, p, stream);
    if (mode == 1) return c3_launch_mode<MT, NT, 1>(a, p, stream);
    return c3_launch_mode<MT, NT, 2>(a, p, stream);
}

} // namespace

// 3x3, stride 1, pad 1, reduced channels a multiple of 64 from 128 up, output channels a multiple of 16 from
// 64 up (forward; the input gradient of such a layer with the roles of C and Cout swapped).
// HQ_E_BADSHAPE: not covered.  force_cfg (testing / tuning): 0 = choose, else 10 * MT + NT.
int hq_try_launch_conv3(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                        const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                        int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed,
                        int force_cfg)
{
    if (sr_seed && out32) return HQ_E_BADARG;
    if (p->kind != HQ_CONV2D || p->R != 3 || p->S != 3 || p->stride != 1 || p->pad != 1) return HQ_E_BADSHAPE;
    const int C = dgrad ? p->Cout : p->C, N = dgrad ? p->C : p->Cout;
    if (C % 64 != 0 || C < 128 || N % 16 != 0 || N < 64) return HQ_E_BADSHAPE;
    const long M = (long)p->B * p->H * p->W;
    const int big = p->W > p->H ? p->W : p->H;
    if ((unsigned long long)M * (unsigned)(big + 2) >= (1ull << 32)) return HQ_E_BADSHAPE;     // hq_magic_div's range
    Conv3Args a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.Bn = p->B; a.H = p->H; a.W = p->W; a.C = C; a.N = N;
    a.flip = dgrad ? 1 : 0;
    a.M = (int)M;
    a.PW = p->W + 2; a.H2 = p->H + 2;
    a.magic_W = hq_magic32((unsigned)p->W); a.magic_H = hq_magic32((unsigned)p->H);
    a.magic_PW = hq_magic32((unsigned)a.PW); a.magic_H2 = hq_magic32((unsigned)a.H2);
    a.count = (unsigned long long)M * N;
    a.sr = sr_seed ? HqSr{(unsigned)*sr_seed, (unsigned)(*sr_seed >> 32)} : HqSr{0, 0};
    const int mode = out32 ? 0 : sr_seed ? 2 : 1;

    // Tile shape: the one that needs the least time by a simple model -- rounds of 256 workgroups times the
    // tile's MFMA work over the efficiency of its wavefront tile -- among those whose LDS fits.
    struct Cfg { int mt, nt; double eff; size_t lds; };
    const Cfg cfgs[4] = {{4, 4, 1.00, c3_lds_bytes<4, 4>(p)}, {4, 2, 0.85, c3_lds_bytes<4, 2>(p)},
                         {2, 4, 0.85, c3_lds_bytes<2, 4>(p)}, {2, 2, 0.70, c3_lds_bytes<2, 2>(p)}};
    int best = -1;
    double best_cost = 0.0;
    for (int i = 0; i < 4; i++) {
        const Cfg &c = cfgs[i];
        if (c.lds > C3_LDS_MAX) continue;
        if (force_cfg && force_cfg != 10 * c.mt + c.nt) continue;
        if (!force_cfg && 64 * c.nt > ((N + 63) / 64) * 64) continue;       // wider than the layer
        const long items = ((M + 64 * c.mt - 1) / (64 * c.mt)) * ((N + 64 * c.nt - 1) / (64 * c.nt));
        const double cost = (double)((items + 255) / 256) * c.mt * c.nt / c.eff;
        if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
    }
    if (best < 0) return HQ_E_BADSHAPE;
    switch (10 * cfgs[best].mt + cfgs[best].nt) {
    case 44: return c3_launch<4, 4>(a, p, mode, stream);
    case 42: return c3_launch<4, 2>(a, p, mode, stream);
    case 24: return c3_launch<2, 4>(a, p, mode, stream);
    default: return c3_launch<2, 2>(a, p, mode, stream);
    }
}
