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

template <int TN, int TK>
__global__ __launch_bounds__(HQ_THREADS) void hq_wgrad_kernel(const WgradArgs a)
{
    constexpr int PG = TN + 32, PX = TK + 32;           // LDS pitches (32 mod 64: best for the transposing reads)
    constexpr int WTN = TN / 2, WTK = TK / 2;           // 2 x 2 wavefronts
    constexpr int NT = WTN / 32, KT = WTK / 32;
    constexpr int GCH = TN / 16, XCH = TK / 16;         // 16-byte chunks per tile row
    constexpr int GLD = MB * GCH / HQ_THREADS, XLD = MB * XCH / HQ_THREADS;
    static_assert(GLD >= 1 && XLD >= 1, "tile too small for 256 loader threads");

    __shared__ __attribute__((aligned(16))) int8_t Gs[2][MB * PG];
    __shared__ __attribute__((aligned(16))) int8_t Xs[2][MB * PX];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    const int tap = bx / a.ctiles, c0 = (bx % a.ctiles) * TK;
    const int tr = tap / a.S, ts = tap % a.S;
    const int n0 = by * TN;
    const int m_begin = bz * a.m_per_split;
    const int m_end = min(a.M, m_begin + a.m_per_split);
    const int zx = a.xq->zero_point;
    const int fill = (zx & 0xff) * 0x01010101;
    const bool do_gsum = bx == 0 && wk == 0;     // column sums of G: first tile column
    const bool do_xsum = by == 0 && wn == 0;     // column sums of Xg: first tile row

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
            if (m < m_end && c < a.C) {
                const int ow = m % a.OW, oh = (m / a.OW) % a.OH, b = m / (a.OW * a.OH);
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
            const int c = c0 + wk * WTK + j * 32 + (lane & 31);
            if (c >= a.C) continue;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int n = n0 + wn * WTN + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (n < a.N && acc[i][j][r] != 0) atomicAdd(a.acc + (size_t)n * krow + (size_t)tap * a.C + c, acc[i][j][r]);
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
            const int c = c0 + wk * WTK + j * 32 + (lane & 31);
            if (lane < 32 && c < a.C && s != 0) atomicAdd(a.xsum + (size_t)tap * a.C + c, s);
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
                                      int gsum_per_k, float *dW, int32_t *dW_acc)
{
    const unsigned zx = (unsigned)xq->zero_point, zg = (unsigned)gq->zero_point;
    const float s = __fmul_rn(xq->scale, gq->scale);
    const size_t total = (size_t)N * K;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int n = (int)(i / K), k = (int)(i % K);
        const unsigned g = (unsigned)gsum[gsum_per_k ? k % gsum_per_k : n];
        unsigned c = (unsigned)acc[i] - zx * g - zg * (unsigned)xsum[k] + M * zx * zg;
        if (dW_acc) dW_acc[i] = (int)c;
        dW[i] = __fmul_rn(s, (float)(int)c);
    }
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

} // namespace

size_t hq_wgrad_workspace_bytes(const hq_problem *p)
{
    const size_t K = (size_t)p->R * p->S * p->C;
    if (p->kind == HQ_DEPTHWISE) return align16(4 * K) + align16(4 * (size_t)p->C) + align16(4 * K);
    return align16(4 * (size_t)p->Cout * K) + align16(4 * (size_t)p->Cout) + align16(4 * K);
}

int hq_launch_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                    const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, hipStream_t stream)
{
    const int OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    const size_t K = (size_t)p->R * p->S * p->C;
    WgradArgs a;
    a.X = X; a.G = dY; a.xq = xq; a.gq = gq;
    char *w = static_cast<char *>(ws);
    a.acc = reinterpret_cast<int32_t *>(w);
    a.gsum = reinterpret_cast<int32_t *>(w + align16(4 * (size_t)p->Cout * K));
    a.xsum = reinterpret_cast<int32_t *>(w + align16(4 * (size_t)p->Cout * K) + align16(4 * (size_t)p->Cout));
    a.M = p->B * OH * OW; a.N = p->Cout; a.C = p->C;
    a.R = p->R; a.S = p->S; a.H = p->H; a.W = p->W; a.OH = OH; a.OW = OW; a.stride = p->stride; a.pad = p->pad;
    a.g16 = (a.N % 16) == 0; a.x16 = (a.C % 16) == 0;

    const size_t ws_words = hq_wgrad_workspace_bytes(p) / 4;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((ws_words + 255) / 256 > 1024 ? 1024 : (ws_words + 255) / 256)),
                       dim3(256), 0, stream, a.acc, ws_words);

    const bool big = a.N > 64 && a.C > 64;
    const int TN = big ? 128 : 64, TK = big ? 128 : 64;
    a.ctiles = (a.C + TK - 1) / TK;
    const int xt = p->R * p->S * a.ctiles, yt = (a.N + TN - 1) / TN;
    const int stages_total = (a.M + MB - 1) / MB;
    int splits = (2048 + xt * yt - 1) / (xt * yt);          // aim at ~8 workgroups per CU
    if (splits > stages_total) splits = stages_total;
    if (splits < 1) splits = 1;
    const int stages_per = (stages_total + splits - 1) / splits;
    a.m_per_split = stages_per * MB;
    splits = (stages_total + stages_per - 1) / stages_per;
    a.xt = xt; a.yt = yt; a.splits = splits;
    dim3 grid((unsigned)(xt * yt * splits));
    if (big) hipLaunchKernelGGL((hq_wgrad_kernel<128, 128>), grid, dim3(HQ_THREADS), 0, stream, a);
    else     hipLaunchKernelGGL((hq_wgrad_kernel<64, 64>), grid, dim3(HQ_THREADS), 0, stream, a);

    const size_t total = (size_t)a.N * K;
    unsigned fb = (unsigned)((total + 255) / 256 > 2048 ? 2048 : (total + 255) / 256);
    hipLaunchKernelGGL(wgrad_finalize_kernel, dim3(fb), dim3(256), 0, stream, a.acc, a.gsum, a.xsum, xq, gq,
                       (unsigned)a.M, a.N, (int)K, 0, dW, dW_acc);
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP;
}
