// 3x3 stride-1 convolution with many channels (C a multiple of 64 from 128 up, Cout a multiple of
// 128) on int8 MFMA with the fused in-hindsight epilogue: forward and, with mirrored taps, the input
// gradient of the layers of ResNet stages 2 to 4 (paper Sec. 3.1; Sec. 3.2 static quantization;
// Sec. 4 steps 1 and 2).
//
// The general gather kernel fetches every input byte once per tap: at a 128x128 tile that is 64
// bytes through the vector memory path per clock of matrix work, which is all that path delivers.
// Here a workgroup stages the input pixels of its tile once per 64-channel chunk, with their
// one-pixel border (zero-point code outside the image), and the nine taps are nine shifted views
// of that patch.  The weights are too large to stay in LDS; they stream through it in stages of one
// (tap, 64-channel chunk): 128 rows of 64 bytes, two buffers.  Everything goes global -> LDS without
// passing through registers (global_load_lds_dwordx4: lane l of a wavefront lands at base + 16 * l),
// so LDS rows are dense and their four 16-byte chunks are XOR-swizzled by the row index, applied to
// the chunk a lane fetches.  A stage of the loop covers two (tap, chunk) steps: one barrier per
// 32 MFMAs of a wavefront.
//
// Tile: up to 256 output pixels (whole rows of one image, or several whole small images) by 128
// output channels; four wavefronts, each 64 pixels x 128 channels (128 accumulators per lane).
#include "hq_device.h"
#include "hq_internal.h"
#include <type_traits>

namespace {

constexpr int BW_BN = 128;         // output channels per item
constexpr int BW_NT = 4;           // 32-channel blocks per wavefront
constexpr int BW_CK = 64;          // channels per reduction chunk (bytes per LDS row)

struct BandwArgs {
    const int8_t *A, *Bw;
    const int32_t *bsum;
    const hq_qparams *aq, *bq;
    const hq_range *range;
    int8_t *out8;
    int32_t *out32;
    hq_qparams *outq;
    hq_stats *st;
    int Bn, H, W, C, N;            // stride 1, "same" size: the output image is H x W
    int pad, flip;                 // effective padding (1 for a 3x3 layer), weight taps mirrored (dgrad)
    int rows, nimg;                // tile: `rows` rows of one image, or `nimg` whole images (rows == H)
    int tiles_per_image;           // nimg == 1: ceil(H / rows)
    int ntiles, nchunks;           // pixel tiles, 128-channel chunks of the output
    int PH, PW;                    // patch rows per image (rows + 2) and patch row length (W + 2)
    int patch_px;                  // nimg * PH * PW
    unsigned magic_img, magic_PW;  // ceil(2^32 / (PH * PW)), ceil(2^32 / PW)
    unsigned magic_HW, magic_W;    // ceil(2^32 / (H * W)), ceil(2^32 / W): a tile pixel -> (image, row, column)
    unsigned long long count;
    HqSr sr;                       // seed of stochastic rounding (epilogue mode 2)
};

// 16-byte rows of one repeated byte value, indexed by that value: the source of the lanes of a direct-to-LDS
// load that lie outside the image (zero-point code) or beyond the weight tensor (0), so that every lane of
// every load has an address and a wavefront's count of outstanding loads does not depend on its data.
struct BwFillRows {
    unsigned w[256][4];
    constexpr BwFillRows() : w()
    {
        for (int v = 0; v < 256; v++)
            for (int k = 0; k < 4; k++) w[v][k] = (unsigned)v * 0x01010101u;
    }
};
__device__ const BwFillRows bw_fill_rows = BwFillRows();

__device__ inline int bw_sigma32(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }
__device__ inline int bw_swz(int row) { return (row >> 2) & 3; }

// MODE: 0 = 32-bit outputs, 1 = fused requantization with round-half-even, 2 = fused with
// stochastic rounding (input gradients).
template <int MODE>
__global__ __launch_bounds__(HQ_THREADS, 2) void hq_bandw_kernel(const BandwArgs a)
{
    constexpr bool FUSED = MODE != 0, SR = MODE == 2;
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    const int patch_bytes = (a.patch_px * BW_CK + 1023) & ~1023;       // whole wavefront loads
    int8_t *Wl = smem;                                     // [2 buffers][2 steps][128][64]
    int8_t *Pl = smem + 4 * BW_BN * BW_CK;                 // [2][patch_px][64]
    int *bz = reinterpret_cast<int *>(Pl + 2 * (size_t)patch_bytes);    // [128]
    int *red = bz + BW_BN;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);         // scalar: branches on it are uniform
    const int za = a.aq->zero_point;
    const int8_t *fill_src = reinterpret_cast<const int8_t *>(bw_fill_rows.w[za & 0xff]);
    const int8_t *zero_src = reinterpret_cast<const int8_t *>(bw_fill_rows.w[0]);
    const float acc_scale = __fmul_rn(a.aq->scale, a.bq->scale);
    HqEpilogue ep = {1.0f, 0.0f, 0.0f, 0.0f, true};
    if (FUSED) ep = hq_make_epilogue(acc_scale, a.range);
    const int cchunks = a.C / BW_CK, nsteps = cchunks * 9, nstages = (nsteps + 1) / 2;
    const size_t wrow = (size_t)9 * a.C;                   // bytes of a weight row

    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;

    for (int item = blockIdx.x; item < a.ntiles * a.nchunks; item += gridDim.x) {
        const int tile = item / a.nchunks, nc = item - tile * a.nchunks;
        const int n0 = nc * BW_BN;
        // ---- the tile's pixels
        int b0, y0, trows, timg;
        if (a.nimg == 1) {
            b0 = tile / a.tiles_per_image; y0 = (tile - b0 * a.tiles_per_image) * a.rows;
            trows = min(a.rows, a.H - y0); timg = 1;
        } else {
            b0 = tile * a.nimg; y0 = 0; trows = a.H; timg = min(a.nimg, a.Bn - b0);
        }
        const int npix = timg * trows * a.W;
        const size_t pix0 = ((size_t)b0 * a.H + y0) * a.W;             // first output pixel (NHWC order)

        __syncthreads();                                   // the previous item's readers are done with bz and LDS
        if (tid < BW_BN) bz[tid] = n0 + tid < a.N ? za * a.bsum[n0 + tid] : 0;

        // ---- loaders.  Patch chunk: LDS slot q -> patch pixel q / 4, 16-byte chunk q % 4 (swizzled source).
        auto issue_patch = [&](int cchunk, int buf) {
            int8_t *dstp = Pl + (size_t)buf * patch_bytes;
            for (int q0 = 0; q0 < a.patch_px * 4; q0 += HQ_THREADS) {
                const int q = q0 + tid;
                const int ppix = q >> 2, ck = (q & 3) ^ bw_swz(ppix);
                const int il = (int)hq_magic_div((unsigned)ppix, a.magic_img), r1 = ppix - il * (a.PH * a.PW);
                const int pr = (int)hq_magic_div((unsigned)r1, a.magic_PW), pc = r1 - pr * a.PW;
                const int iy = y0 + pr - a.pad, ix = pc - a.pad;
                const bool inside = q < a.patch_px * 4 && il < timg && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                int8_t *dst = dstp + (size_t)(q0 + wave * 64) * 16;     // this wavefront's 1 KiB
                if (q0 + wave * 64 < a.patch_px * 4) {                  // (uniform over the wavefront)
                    const int8_t *src = a.A + (((size_t)(b0 + il) * a.H + iy) * a.W + ix) * a.C + cchunk * BW_CK + ck * 16;
                    hq_global_to_lds16(inside ? src : fill_src, dst);
                }
            }
        };
        // Weight stage (two steps): LDS row = channel sigma-permuted inside its 32-block, slot q -> row q / 4,
        // chunk q % 4.
        const int8_t *wsrc[2];                             // this thread's two weight rows, at its (swizzled) chunk
        bool wrow_ok[2];
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const int q = tid + HQ_THREADS * k, row = q >> 2, ck = (q & 3) ^ bw_swz(row);
            const int n = n0 + (row & ~31) + bw_sigma32(row & 31);
            wrow_ok[k] = n < a.N;
            wsrc[k] = a.Bw + (size_t)(wrow_ok[k] ? n : 0) * wrow + ck * 16;
        }
        // The weights go through registers (two steps = four 16-byte loads per thread, requested at the start of a
        // stage, written to LDS at its end): the direct-to-LDS path moves about 20 bytes per clock and compute
        // unit, register loads 30 to 35, and a stage of two workgroups needs 32 KB of weights per 2048 clocks.
        v4i wreg[2][2];
        auto load_weights = [&](int stage) {
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int step = min(2 * stage + u, nsteps - 1);
                const bool real = 2 * stage + u < nsteps;              // an odd count of steps ends on a step of zero weights
                const int cchunk = step / 9, tap = step - cchunk * 9;
                const int woff = (a.flip ? 8 - tap : tap) * a.C + cchunk * BW_CK;
#pragma unroll
                for (int k = 0; k < 2; k++)
                    wreg[u][k] = *(const __attribute__((address_space(1))) v4i *)(wrow_ok[k] && real ? wsrc[k] + woff : zero_src);
            }
        };
        auto store_weights = [&](int buf) {
#pragma unroll
            for (int u = 0; u < 2; u++)
#pragma unroll
                for (int k = 0; k < 2; k++)
                    *reinterpret_cast<v4i *>(Wl + (size_t)(buf * 2 + u) * BW_BN * BW_CK + (size_t)(HQ_THREADS * k + tid) * 16) = wreg[u][k];
        };

        issue_patch(0, 0);
        load_weights(0);
        store_weights(0);

        // ---- this lane's two pixels: patch row of tap (0, 0), and whether they exist
        int prow[2];
        bool ok[2];
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int pt = wave * 64 + i * 32 + (lane & 31);
            ok[i] = pt < npix;
            const int p = ok[i] ? pt : 0;
            // (tiles of several images hold whole images: trows == H there; p < 256)
            const int il = a.nimg == 1 ? 0 : (int)hq_magic_div((unsigned)p, a.magic_HW), r1 = p - il * (trows * a.W);
            const int oy = (int)hq_magic_div((unsigned)r1, a.magic_W), ox = r1 - oy * a.W;
            prow[i] = (il * a.PH + oy) * a.PW + ox;
        }
        const bool active = wave * 64 < npix;                          // scalar
        int wfoff[2];                                      // weight fragment offset of k-step ks in 32-row block 0
#pragma unroll                                             // (the swizzle repeats every 8 rows: block j adds j * 2048)
        for (int ks = 0; ks < 2; ks++)
            wfoff[ks] = (lane & 31) * BW_CK + 16 * ((2 * ks + half) ^ bw_swz(lane & 31));

        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        v16i acc[2][BW_NT];
#pragma unroll
        for (int j = 0; j < BW_NT; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const v4i bzv = *reinterpret_cast<const v4i *>(bz + j * 32 + 16 * half + 4 * g);
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[i][j][4 * g + e] = -bzv[e];
            }

        for (int s = 0; s < nstages; s++) {
            // four k-steps (two per (tap, chunk) step) with two fragment register sets: the fragments of
            // k-step kk + 1 are requested before the MFMAs of k-step kk are issued, and the stage's first
            // fragments before the next stage's loads, whose address arithmetic then runs under their latency
            const int c0 = (2 * s) / 9, t0 = 2 * s - c0 * 9;
            // the next chunk's patch is requested by the first stage that lies wholly inside this chunk:
            // every reader of the buffer it overwrites finished before that stage's opening barrier
            const bool patch_now = t0 <= 1 && c0 + 1 < cchunks;
            const int8_t *Wb[2], *Pb[2];
            int toff[2];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int step = min(2 * s + u, nsteps - 1);
                const int cchunk = step / 9, tap = step - cchunk * 9;
                Wb[u] = Wl + (size_t)((s & 1) * 2 + u) * BW_BN * BW_CK;
                Pb[u] = Pl + (size_t)(cchunk & 1) * patch_bytes;
                toff[u] = (tap / 3) * a.PW + (tap % 3);
            }
            v4i wfA[BW_NT], afA[2], wfB[BW_NT], afB[2];
            auto load_frags = [&](int kk, v4i (&wf)[BW_NT], v4i (&af)[2]) {
                const int u = kk >> 1, ks = kk & 1;
#pragma unroll
                for (int j = 0; j < BW_NT; j++) wf[j] = *reinterpret_cast<const v4i *>(Wb[u] + j * 32 * BW_CK + wfoff[ks]);
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    const int row = prow[i] + toff[u];
                    af[i] = *reinterpret_cast<const v4i *>(Pb[u] + row * BW_CK + 16 * ((2 * ks + half) ^ bw_swz(row)));
                }
            };
            auto mfmas = [&](const v4i (&wf)[BW_NT], const v4i (&af)[2]) {
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int j = 0; j < BW_NT; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], acc[i][j], 0, 0, 0);
            };
            if (s + 1 < nstages) load_weights(s + 1);
            if (active) {
                // the fragment reads of k-step kk + 1 and their address arithmetic are dealt between the MFMAs of
                // k-step kk (a wavefront issues in order: an MFMA holds the matrix pipe for 32 cycles, in which it
                // can issue seven other instructions)
                auto interleave = [&]() {
#pragma unroll
                    for (int q = 0; q < 6; q++) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);     // two vector ALU instructions
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                };
                load_frags(0, wfA, afA);
                if (patch_now) issue_patch(c0 + 1, (c0 + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                load_frags(1, wfB, afB);
                mfmas(wfA, afA);
                interleave();
                __builtin_amdgcn_sched_barrier(0);
                load_frags(2, wfA, afA);
                mfmas(wfB, afB);
                interleave();
                __builtin_amdgcn_sched_barrier(0);
                load_frags(3, wfB, afB);
                mfmas(wfA, afA);
                interleave();
                __builtin_amdgcn_sched_barrier(0);
                mfmas(wfB, afB);
            } else {
                if (patch_now) issue_patch(c0 + 1, (c0 + 1) & 1);
            }
            // the other weight buffer was last read in the previous stage, behind whose barrier every wavefront is
            if (s + 1 < nstages) store_weights((s + 1) & 1);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }

        // ---- epilogue: lane = one pixel per 32-row block, 16 consecutive channels per column block
        auto epilogue = [&](auto full) {
            constexpr bool FULL = decltype(full)::value;
#pragma unroll
            for (int i = 0; i < 2; i++) {
                if (!ok[i]) continue;
                const size_t m = pix0 + wave * 64 + i * 32 + (lane & 31);
#pragma unroll
                for (int j = 0; j < BW_NT; j++) {
                    const int nb = n0 + j * 32 + 16 * half;
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

} // namespace

// 3x3, stride 1, pad 1, C % 64 == 0 and C >= 128, Cout % 16 == 0 and Cout >= 128 (forward); the
// input gradient of such a layer with the roles of C and Cout swapped.  HQ_E_BADSHAPE: not covered.
int hq_try_launch_bandw(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                        const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                        int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed)
{
    if (sr_seed && out32) return HQ_E_BADARG;
    if (p->kind != HQ_CONV2D || p->R != 3 || p->S != 3 || p->stride != 1 || p->pad != 1) return HQ_E_BADSHAPE;
    const int C = dgrad ? p->Cout : p->C, N = dgrad ? p->C : p->Cout;
    if (C % 64 != 0 || C < 128 || N % 16 != 0 || N < 128) return HQ_E_BADSHAPE;
    BandwArgs a;
    a.A = A; a.Bw = Bw; a.bsum = bsum; a.aq = aq; a.bq = bq; a.range = range;
    a.out8 = out8; a.out32 = out32; a.outq = outq; a.st = st;
    a.Bn = p->B; a.H = p->H; a.W = p->W; a.C = C; a.N = N;
    a.pad = 1; a.flip = dgrad ? 1 : 0;
    if (p->H * p->W >= 256 || p->H * p->W * 2 > 256) {
        a.nimg = 1;
        a.rows = 256 / p->W < 1 ? 0 : 256 / p->W;
        if (a.rows > p->H) a.rows = p->H;
        if (a.rows < 1) return HQ_E_BADSHAPE;
    } else {
        a.nimg = 256 / (p->H * p->W);
        a.rows = p->H;
    }
    a.tiles_per_image = (p->H + a.rows - 1) / a.rows;
    a.ntiles = a.nimg == 1 ? p->B * a.tiles_per_image : (p->B + a.nimg - 1) / a.nimg;
    a.nchunks = (N + BW_BN - 1) / BW_BN;
    a.PH = a.rows + 2; a.PW = p->W + 2;
    a.patch_px = a.nimg * a.PH * a.PW;
    a.magic_img = hq_magic32((unsigned)(a.PH * a.PW));
    a.magic_PW = hq_magic32((unsigned)a.PW);
    a.magic_HW = hq_magic32((unsigned)(p->H * p->W));
    a.magic_W = hq_magic32((unsigned)p->W);
    a.count = (unsigned long long)p->B * p->H * p->W * N;
    a.sr = sr_seed ? HqSr{(unsigned)*sr_seed, (unsigned)(*sr_seed >> 32)} : HqSr{0, 0};
    const size_t patch_bytes = ((size_t)a.patch_px * BW_CK + 1023) & ~(size_t)1023;
    const size_t lds = 4 * BW_BN * BW_CK + 2 * patch_bytes + 4 * BW_BN + 64;
    if (lds > 158 * 1024) return HQ_E_BADSHAPE;            // (two workgroups per compute unit up to 78 KiB)
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(hq_bandw_kernel<0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(hq_bandw_kernel<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(hq_bandw_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return HQ_E_HIP;
        configured = true;
    }
    long items = (long)a.ntiles * a.nchunks;
    // Too few tiles for the chip under a reduction long enough to matter (4 x 4 images with 512 channels):
    // the gather kernel's 64 x 64 tiles spread the same work over four times as many workgroups.
    if (items < 192 && (unsigned long long)a.count * 9ull * (unsigned)C >= (1ull << 32)) return HQ_E_BADSHAPE;
    const int blocks = (int)(items < 512 ? items : 512);
    if (out32 != nullptr) hipLaunchKernelGGL(hq_bandw_kernel<0>, dim3(blocks), dim3(HQ_THREADS), lds, stream, a);
    else if (sr_seed)     hipLaunchKernelGGL(hq_bandw_kernel<2>, dim3(blocks), dim3(HQ_THREADS), lds, stream, a);
    else                  hipLaunchKernelGGL(hq_bandw_kernel<1>, dim3(blocks), dim3(HQ_THREADS), lds, stream, a);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}
