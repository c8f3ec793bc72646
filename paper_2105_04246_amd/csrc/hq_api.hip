// C-ABI entry points of the hq library: argument checks, dispatch, and the small kernels
// around the GEMMs (range update, statistics reset, dynamic-baseline middle and second
// pass, weight-side preparation).
#include "hq_device.h"
#include "hq_internal.h"

#include <mutex>

// Scratch memory of hq_gemm_wgrad_static: one array per GPU, held from the moment the library is
// loaded on that GPU until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and launchers receive the device address that call returns.
static __device__ __align__(256) unsigned char hq_static_scratch[HQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int HQ_MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[HQ_MAX_DEVICES];           // device address of hq_static_scratch on each GPU, once resolved

// Device address of the current GPU's copy of the scratch array (resolved on the first call per GPU).
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= HQ_MAX_DEVICES) return HQ_E_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(hq_static_scratch)) != hipSuccess || !ptr) return HQ_E_HIP;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return HQ_OK;
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP; }

// Empties a record; called by the 64 lanes of one wavefront (lane = partial record).
__device__ inline void stats_clear_wave(hq_stats *st)
{
    const int lane = threadIdx.x & 63;
    hq_stats_part *p = &st->part[lane];
    p->acc_min = INT_MAX; p->acc_max = INT_MIN; p->clip_lo = 0; p->clip_hi = 0;
    if (lane == 0) {
        st->acc_min = INT_MAX; st->acc_max = INT_MIN; st->acc_scale = 0.0f; st->fp32_keys = 0;
        st->clip_lo = 0; st->clip_hi = 0; st->count = 0;
    }
}

__global__ __launch_bounds__(64) void range_update_kernel(hq_range *r, hq_stats *st)
{
    hq_range_update_wave(r + blockIdx.x, st + blockIdx.x);
}

// Saturation-driven update of one quantizer per workgroup (one wavefront): folds the statistics, moves the
// range by the rule stated with hq_range_update_saturation, empties the record.
__global__ __launch_bounds__(64) void range_update_saturation_kernel(hq_range *r, hq_stats *st, hq_saturation *sat)
{
    r += blockIdx.x; st += blockIdx.x; sat += blockIdx.x;
    hq_range rr = *r;
    hq_saturation ss = *sat;
    const float acc_scale = st->acc_scale;
    const unsigned long long count = st->count;
    const HqStatsFolded f = hq_stats_fold_wave(st);
    if (threadIdx.x == 0) {
        if (count != 0) {
            hq_saturation_update(&rr, &ss, f.clip_lo + f.clip_hi, count,
                                 __fmul_rn(acc_scale, (float)f.acc_min), __fmul_rn(acc_scale, (float)f.acc_max));
            *r = rr; *sat = ss;
        }
        st->acc_min = INT_MAX; st->acc_max = INT_MIN; st->acc_scale = 0.0f; st->fp32_keys = 0;
        st->clip_lo = 0; st->clip_hi = 0; st->count = 0;
    }
}

__global__ __launch_bounds__(64) void stats_reset_kernel(hq_stats *st) { stats_clear_wave(st + blockIdx.x); }

__global__ __launch_bounds__(64) void stats_fold_kernel(hq_stats *st) { hq_stats_fold_wave(st + blockIdx.x); }

// Dynamic baseline, between the passes: the quantizer of the tensor just written.
__global__ __launch_bounds__(64) void dynamic_mid_kernel(int mode, hq_range *r, hq_stats *st, hq_qparams *outq)
{
    const HqStatsFolded f = hq_stats_fold_wave(st);
    if (threadIdx.x != 0) return;
    const float gmin = __fmul_rn(st->acc_scale, (float)f.acc_min);
    const float gmax = __fmul_rn(st->acc_scale, (float)f.acc_max);
    if (mode == HQ_DYN_RUNNING) {
        hq_ema_update(r, gmin, gmax);                 // running min-max: this tensor moves the range first
        *outq = r->qp;
    } else {
        if (!r->initialized) hq_ema_update(r, gmin, gmax);          // q^0 = min-max of the first batch
        *outq = hq_qparams_from_range(gmin, gmax, r->symmetric, r->qlo, r->qhi);   // eq. (1)
    }
}

// Dynamic baseline, pass 2: load the 32-bit outputs back (the accumulator-load term of eq. (5)),
// quantize, store codes.  16 outputs per thread: 64 B in, 16 B out.
// SR: stochastic rounding, the draw keyed on the element's index in the output tensor and the seed.
template <bool SR>
__global__ __launch_bounds__(HQ_THREADS) void dynamic_pass2_kernel(const int32_t *__restrict__ c, size_t n,
                                                                   const hq_stats *st, const hq_range *r,
                                                                   const hq_qparams *outq, int8_t *__restrict__ out,
                                                                   hq_stats *st_out, HqSr sr)
{
    __shared__ int red[4 * (HQ_THREADS / 64)];
    const HqRequant rq = hq_make_requant(st->acc_scale, *outq, r->qlo, r->qhi);
    unsigned nlo = 0, nhi = 0;
    auto one = [&](int v, size_t idx) __attribute__((always_inline)) -> int {
        return SR ? hq_requant_sr(v, rq, sr, idx, nlo, nhi) : hq_requant(v, rq, nlo, nhi);
    };
    const size_t groups = n / 16, step = (size_t)gridDim.x * blockDim.x;
    for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += step) {
        const v4i *src = reinterpret_cast<const v4i *>(c) + 4 * g;
        v4i packed;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            v4i v = src[k];
            const size_t i0 = 16 * g + 4 * k;
            packed[k] = (int)hq_pack4(one(v[0], i0), one(v[1], i0 + 1), one(v[2], i0 + 2), one(v[3], i0 + 3));
        }
        reinterpret_cast<v4i *>(out)[g] = packed;
    }
    // tail (n % 16 elements), one thread
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (size_t i = groups * 16; i < n; i++) out[i] = (int8_t)one(c[i], i);
    hq_block_stats_commit(INT_MAX, INT_MIN, nlo, nhi, st_out, red);
}

// Weight-side preparation: per-output-channel and per-input-channel code sums and the
// [C][R][S][Cout] re-layout.  Small tensors, run once per weight update: plain kernels.
__global__ void weight_rowsum_kernel(const int8_t *W, int rows, int len, int32_t *sum)
{
    // one wavefront per row
    int row = blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= rows) return;
    int s = 0;
    for (int i = lane; i < len; i += 64) s += W[(size_t)row * len + i];
    s = hq_wave_reduce(s, HqAdd());
    if (lane == 0) sum[row] = s;
}

__global__ void weight_colsum_kernel(const int8_t *W, int rows, int taps, int C, int32_t *sum)
{
    // sum over (row, tap) for each channel c of W[rows][taps][C]: a workgroup takes a slab of 64
    // (row, tap) lines, a thread one channel of it; the slabs meet with one atomic per channel
    // (sum is zeroed before the launch)
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const int lines = rows * taps, l0 = blockIdx.y * 64, l1 = min(lines, l0 + 64);
    int s = 0;
    for (int i = l0; i < l1; i++) s += W[(size_t)i * C + c];
    if (s != 0) atomicAdd(sum + c, s);
}

__global__ void zero_words_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ void weight_relayout_kernel(const int8_t *W, int Cout, int taps, int C, int8_t *Wd)
{
    // Wd[c][tap][n] = W[n][tap][c]
    size_t total = (size_t)Cout * taps * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int n = (int)(i % Cout); size_t t = i / Cout; int tap = (int)(t % taps); int c = (int)(t / taps);
        Wd[i] = W[((size_t)n * taps + tap) * C + c];
    }
}

// ---------------------------------------------------------------------------------------
// Argument checks
// ---------------------------------------------------------------------------------------
int check_problem(const hq_problem *p)
{
    if (!p) return HQ_E_BADARG;
    if (p->kind != HQ_LINEAR && p->kind != HQ_CONV2D && p->kind != HQ_DEPTHWISE) return HQ_E_BADARG;
    if (p->B <= 0 || p->H <= 0 || p->W <= 0 || p->C <= 0 || p->Cout <= 0 || p->R <= 0 || p->S <= 0 ||
        p->stride <= 0 || p->pad < 0) return HQ_E_BADSHAPE;
    if (p->kind == HQ_LINEAR && (p->H != 1 || p->W != 1 || p->R != 1 || p->S != 1 || p->stride != 1 || p->pad != 0))
        return HQ_E_BADSHAPE;
    if (p->kind == HQ_DEPTHWISE && p->Cout != p->C) return HQ_E_BADSHAPE;
    if (p->H + 2 * p->pad < p->R || p->W + 2 * p->pad < p->S) return HQ_E_BADSHAPE;
    if (p->pad >= p->R || p->pad >= p->S) return HQ_E_BADSHAPE;       // every output has a real tap
    // channel counts are multiples of 4, except that a convolution may read 3-channel (RGB) inputs
    if (((p->C % 4) != 0 && !(p->kind == HQ_CONV2D && p->C == 3)) || (p->Cout % 4) != 0) return HQ_E_BADSHAPE;
    const long OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    const long lim = 0x7fffffffL;
    if ((long)p->B * p->H * p->W >= lim || (long)p->B * OH * OW >= lim) return HQ_E_BADSHAPE;
    if ((long)p->B * p->H * p->W * p->C >= lim * 2 || (long)p->B * OH * OW * p->Cout >= lim * 2) return HQ_E_BADSHAPE;
    if ((long)p->R * p->S * p->C * (p->kind == HQ_DEPTHWISE ? 1 : p->Cout) >= lim) return HQ_E_BADSHAPE;
    return HQ_OK;
}

size_t out_elems(const hq_problem *p, bool dgrad)
{
    const size_t OH = (p->H + 2 * p->pad - p->R) / p->stride + 1, OW = (p->W + 2 * p->pad - p->S) / p->stride + 1;
    return dgrad ? (size_t)p->B * p->H * p->W * p->C : (size_t)p->B * OH * OW * p->Cout;
}

// Q_W: |w| maximum of an FP32 tensor into *bits (non-negative floats order like their bit patterns).
__global__ __launch_bounds__(HQ_THREADS) void weight_absmax_kernel(const float *__restrict__ w, size_t n, unsigned *bits)
{
    __shared__ unsigned red[HQ_THREADS / 64];
    unsigned m = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        m = max(m, __float_as_uint(fabsf(w[i])));
#pragma unroll
    for (int k = 32; k >= 1; k >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, k));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < HQ_THREADS / 64; k++) m = max(m, red[k]);
        if (m) atomicMax(bits, m);
    }
}

__global__ void weight_scale_init_kernel(hq_qparams *wq) { wq->zero_point = 0; }      // the maximum is gathered in this field

__global__ void weight_scale_kernel(hq_qparams *wq)
{
    const float amax = __uint_as_float((unsigned)wq->zero_point);
    wq->scale = amax > 0.0f ? __fdiv_rn(amax, 127.0f) : 1.0f;
    wq->zero_point = 0;
}

__global__ __launch_bounds__(HQ_THREADS) void weight_quantize_kernel(const float *__restrict__ w, size_t n,
                                                                     const hq_qparams *wq, int8_t *__restrict__ out)
{
    const float s = wq->scale;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const float r = fminf(fmaxf(rintf(__fdiv_rn(w[i], s)), -127.0f), 127.0f);
        out[i] = (int8_t)(int)r;
    }
}

// Register-only int8 MFMA loop: eight independent accumulator chains per wavefront, so that the
// matrix pipeline never waits on a dependent result.
__global__ __launch_bounds__(HQ_THREADS) void mfma_rate_kernel(int iters, int32_t *sink)
{
    const int tid = threadIdx.x;
    v4i a = {tid, tid * 3, tid * 5, tid * 7}, b = {tid ^ 0x55, tid + 1, tid + 2, tid + 3};
    v16i acc[8];
#pragma unroll
    for (int j = 0; j < 8; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[j][e] = 0;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 8; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) s ^= acc[j][e];
    sink[(size_t)blockIdx.x * HQ_THREADS + tid] = s;
}

} // namespace

extern "C" {

const char *hq_error_string(int code)
{
    switch (code) {
    case HQ_OK: return "ok";
    case HQ_E_BADARG: return "bad argument (null or misaligned pointer, bad enum)";
    case HQ_E_BADSHAPE: return "unsupported shape";
    case HQ_E_WORKSPACE: return "workspace missing, too small, or (static variant) problem beyond the built-in scratch";
    case HQ_E_HIP: return "HIP launch failed";
    default: return "unknown hq error code";
    }
}

size_t hq_workspace_bytes(int32_t entry, const hq_problem *p)
{
    if (check_problem(p) != HQ_OK) return 0;
    switch (entry) {
    case HQ_ENTRY_WGRAD: return hq_wgrad_workspace_bytes(p);
    case HQ_ENTRY_DYNAMIC_FWD: return 4 * out_elems(p, false);
    case HQ_ENTRY_DYNAMIC_DGRAD: return 4 * out_elems(p, true);
    default: return 0;
    }
}

static int gemm_common(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                       const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out,
                       int32_t *out32, hq_qparams *outq, hq_stats *st, void *stream, const uint64_t *sr_seed = nullptr)
{
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!A || !aq || !Bw || !bq || !bsum || !range || !st || (!out && !out32) || (out && !outq)) return HQ_E_BADARG;
    if (misaligned(A, 16) || misaligned(Bw, 16) || misaligned(bsum, 16) || misaligned(out, 16) ||
        misaligned(out32, 16) || misaligned(st, 128) || misaligned(range, 4) || misaligned(aq, 4) ||
        misaligned(bq, 4) || misaligned(outq, 4)) return HQ_E_BADARG;
    if (p->C == 3) {
        // 3-channel input: the first-layer kernel or nothing (a network's first layer needs no input gradient)
        if (dgrad || sr_seed) return HQ_E_BADSHAPE;
        return hq_try_launch_direct(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
    }
    if (sr_seed) {
        // stochastic rounding: the two 3x3 / 1x1 fast paths, else the two general kernels
        if (p->kind == HQ_DEPTHWISE)
            return hq_launch_depthwise(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream), sr_seed);
        rc = hq_try_launch_bandw(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream), sr_seed);
        if (rc != HQ_E_BADSHAPE) return rc;
        rc = hq_try_launch_band(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream), sr_seed);
        if (rc != HQ_E_BADSHAPE) return rc;
        return hq_launch_gemm(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream), sr_seed);
    }
    if (p->kind == HQ_DEPTHWISE)
        return hq_launch_depthwise(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
    rc = hq_try_launch_direct(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
    if (rc != HQ_E_BADSHAPE) return rc;
    rc = hq_try_launch_bandw(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
    if (rc != HQ_E_BADSHAPE) return rc;
    rc = hq_try_launch_band(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
    if (rc != HQ_E_BADSHAPE) return rc;
    return hq_launch_gemm(p, dgrad, A, aq, Bw, bq, bsum, range, out, out32, outq, st, as_stream(stream));
}

int hq_gemm_fwd(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *W, const hq_qparams *wq,
                const int32_t *wsum, const hq_range *yr, int8_t *Y, hq_qparams *yq, hq_stats *st, void *stream)
{
    return gemm_common(p, 0, X, xq, W, wq, wsum, yr, Y, nullptr, yq, st, stream);
}

int hq_gemm_dgrad(const hq_problem *p, const int8_t *dY, const hq_qparams *gq, const int8_t *Wd, const hq_qparams *wq,
                  const int32_t *wdsum, const hq_range *gr, int8_t *dX, hq_qparams *dxq, hq_stats *st, void *stream)
{
    return gemm_common(p, 1, dY, gq, Wd, wq, wdsum, gr, dX, nullptr, dxq, st, stream);
}

int hq_gemm_dgrad_sr(const hq_problem *p, const int8_t *dY, const hq_qparams *gq, const int8_t *Wd, const hq_qparams *wq,
                     const int32_t *wdsum, const hq_range *gr, uint64_t seed, int8_t *dX, hq_qparams *dxq, hq_stats *st,
                     void *stream)
{
    return gemm_common(p, 1, dY, gq, Wd, wq, wdsum, gr, dX, nullptr, dxq, st, stream, &seed);
}

int hq_gemm_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY, const hq_qparams *gq,
                  float *dW, int32_t *dW_acc, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!X || !xq || !dY || !gq || !dW) return HQ_E_BADARG;
    if (misaligned(X, 16) || misaligned(dY, 16) || misaligned(dW, 16) || misaligned(dW_acc, 16) ||
        misaligned(xq, 4) || misaligned(gq, 4)) return HQ_E_BADARG;
    if (p->C == 3 && p->S * 3 > 32) return HQ_E_BADSHAPE;     // 3-channel inputs: a filter row fits 32 bytes
    const size_t need = hq_wgrad_workspace_bytes(p);
    if (need && (!ws || ws_bytes < need || misaligned(ws, 16))) return HQ_E_WORKSPACE;
    if (p->kind == HQ_DEPTHWISE)
        return hq_launch_depthwise_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, as_stream(stream));
    return hq_launch_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, as_stream(stream));
}

int hq_gemm_wgrad_static(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                         const hq_qparams *gq, float *dW, int32_t *dW_acc, void *stream)
{
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!X || !xq || !dY || !gq || !dW) return HQ_E_BADARG;
    if (hq_wgrad_workspace_bytes(p) > (size_t)HQ_STATIC_SCRATCH_BYTES) return HQ_E_WORKSPACE;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != HQ_OK) return rc;
    return hq_gemm_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, (size_t)HQ_STATIC_SCRATCH_BYTES, stream);
}

int hq_gemm_wgrad_update(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                         const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, size_t ws_bytes,
                         hq_range *r, hq_stats *st, int32_t n, void *stream)
{
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!X || !xq || !dY || !gq || !dW || !r || !st || n < 1 || n > 4096) return HQ_E_BADARG;
    if (misaligned(X, 16) || misaligned(dY, 16) || misaligned(dW, 16) || misaligned(dW_acc, 16) ||
        misaligned(xq, 4) || misaligned(gq, 4) || misaligned(r, 4) || misaligned(st, 128)) return HQ_E_BADARG;
    if (p->C == 3 && p->S * 3 > 32) return HQ_E_BADSHAPE;
    const size_t need = hq_wgrad_workspace_bytes(p);
    if (need && (!ws || ws_bytes < need || misaligned(ws, 16))) return HQ_E_WORKSPACE;
    const HqRideAlong ra = {r, st, n, 0};
    if (p->kind == HQ_DEPTHWISE)
        return hq_launch_depthwise_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, as_stream(stream), &ra);
    return hq_launch_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, as_stream(stream), &ra);
}

int hq_range_update(hq_range *r, hq_stats *st, void *stream)
{
    if (!r || !st || misaligned(r, 4) || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL(range_update_kernel, dim3(1), dim3(64), 0, as_stream(stream), r, st);
    return launch_status();
}

int hq_range_update_batch(hq_range *r, hq_stats *st, int32_t n, void *stream)
{
    if (!r || !st || n <= 0 || misaligned(r, 4) || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL(range_update_kernel, dim3(n), dim3(64), 0, as_stream(stream), r, st);
    return launch_status();
}

int hq_range_update_saturation(hq_range *r, hq_stats *st, hq_saturation *sat, int32_t n, void *stream)
{
    if (!r || !st || !sat || n <= 0 || misaligned(r, 4) || misaligned(st, 128) || misaligned(sat, 4)) return HQ_E_BADARG;
    hipLaunchKernelGGL(range_update_saturation_kernel, dim3(n), dim3(64), 0, as_stream(stream), r, st, sat);
    return launch_status();
}

int hq_stats_reset(hq_stats *st, int32_t n, void *stream)
{
    if (!st || n <= 0 || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL(stats_reset_kernel, dim3(n), dim3(64), 0, as_stream(stream), st);
    return launch_status();
}

int hq_stats_fold(hq_stats *st, int32_t n, void *stream)
{
    if (!st || n <= 0 || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL(stats_fold_kernel, dim3(n), dim3(64), 0, as_stream(stream), st);
    return launch_status();
}

static int dynamic_common(int32_t op, int32_t mode, const hq_problem *p, const int8_t *A, const hq_qparams *aq,
                          const int8_t *Bw, const hq_qparams *bq, const int32_t *bsum, hq_range *r, int8_t *out,
                          hq_qparams *outq, hq_stats *st, void *ws, size_t ws_bytes, void *stream, const uint64_t *sr_seed)
{
    if (op != HQ_ENTRY_DYNAMIC_FWD && op != HQ_ENTRY_DYNAMIC_DGRAD) return HQ_E_BADARG;
    if (mode != HQ_DYN_CURRENT && mode != HQ_DYN_RUNNING) return HQ_E_BADARG;
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!out || !outq || !r) return HQ_E_BADARG;
    const bool dgrad = op == HQ_ENTRY_DYNAMIC_DGRAD;
    const size_t n = out_elems(p, dgrad);
    if (!ws || ws_bytes < 4 * n || misaligned(ws, 16)) return HQ_E_WORKSPACE;
    int32_t *c32 = static_cast<int32_t *>(ws);
    // pass 1: GEMM, 32-bit outputs to memory, min/max on the way
    rc = gemm_common(p, dgrad ? 1 : 0, A, aq, Bw, bq, bsum, r, nullptr, c32, outq, st, stream);
    if (rc != HQ_OK) return rc;
    hipLaunchKernelGGL(dynamic_mid_kernel, dim3(1), dim3(64), 0, as_stream(stream), mode, r, st, outq);
    // pass 2: read back, quantize, store codes
    size_t groups = n / 16;
    unsigned blocks = (unsigned)((groups + HQ_THREADS - 1) / HQ_THREADS);
    if (blocks < 1) blocks = 1;
    if (blocks > 256u * 16u) blocks = 256u * 16u;
    if (sr_seed)
        hipLaunchKernelGGL(dynamic_pass2_kernel<true>, dim3(blocks), dim3(HQ_THREADS), 0, as_stream(stream),
                           c32, n, st, r, outq, out, st, HqSr{(unsigned)*sr_seed, (unsigned)(*sr_seed >> 32)});
    else
        hipLaunchKernelGGL(dynamic_pass2_kernel<false>, dim3(blocks), dim3(HQ_THREADS), 0, as_stream(stream),
                           c32, n, st, r, outq, out, st, HqSr{0, 0});
    return launch_status();
}

int hq_gemm_dynamic(int32_t op, int32_t mode, const hq_problem *p, const int8_t *A, const hq_qparams *aq,
                    const int8_t *Bw, const hq_qparams *bq, const int32_t *bsum, hq_range *r, int8_t *out,
                    hq_qparams *outq, hq_stats *st, void *ws, size_t ws_bytes, void *stream)
{
    return dynamic_common(op, mode, p, A, aq, Bw, bq, bsum, r, out, outq, st, ws, ws_bytes, stream, nullptr);
}

int hq_gemm_dynamic_sr(int32_t op, int32_t mode, const hq_problem *p, const int8_t *A, const hq_qparams *aq,
                       const int8_t *Bw, const hq_qparams *bq, const int32_t *bsum, hq_range *r, uint64_t seed,
                       int8_t *out, hq_qparams *outq, hq_stats *st, void *ws, size_t ws_bytes, void *stream)
{
    return dynamic_common(op, mode, p, A, aq, Bw, bq, bsum, r, out, outq, st, ws, ws_bytes, stream, &seed);
}

int hq_weight_prepare(const hq_problem *p, const int8_t *W, int8_t *Wd, int32_t *wsum, int32_t *wdsum, void *stream)
{
    int rc = check_problem(p);
    if (rc != HQ_OK) return rc;
    if (!W) return HQ_E_BADARG;
    hipStream_t s = as_stream(stream);
    const int taps = p->R * p->S;
    auto colsum = [&](int rows, int32_t *sum) {
        hipLaunchKernelGGL(zero_words_kernel, dim3((p->C + 255) / 256), dim3(256), 0, s, sum, p->C);
        hipLaunchKernelGGL(weight_colsum_kernel, dim3((p->C + 63) / 64, (rows * taps + 63) / 64), dim3(64), 0, s,
                           W, rows, taps, p->C, sum);
    };
    if (p->kind == HQ_DEPTHWISE) {
        if (wsum) colsum(1, wsum);
        if (wdsum) colsum(1, wdsum);
        return launch_status();
    }
    if (wsum) hipLaunchKernelGGL(weight_rowsum_kernel, dim3((p->Cout + 3) / 4), dim3(256), 0, s, W, p->Cout, taps * p->C, wsum);
    if (wdsum) colsum(p->Cout, wdsum);
    if (Wd) hipLaunchKernelGGL(weight_relayout_kernel, dim3(1024), dim3(256), 0, s, W, p->Cout, taps, p->C, Wd);
    return launch_status();
}

int hq_weight_quantize(const float *Wf, size_t n, int8_t *Wq, hq_qparams *wq, void *stream)
{
    if (!Wf || !Wq || !wq || n == 0 || misaligned(Wf, 4) || misaligned(wq, 4)) return HQ_E_BADARG;
    hipStream_t s = as_stream(stream);
    size_t blocks = (n + HQ_THREADS - 1) / HQ_THREADS;
    if (blocks > 256u * 16u) blocks = 256u * 16u;
    hipLaunchKernelGGL(weight_scale_init_kernel, dim3(1), dim3(1), 0, s, wq);
    hipLaunchKernelGGL(weight_absmax_kernel, dim3((unsigned)blocks), dim3(HQ_THREADS), 0, s, Wf, n,
                       reinterpret_cast<unsigned *>(&wq->zero_point));
    hipLaunchKernelGGL(weight_scale_kernel, dim3(1), dim3(1), 0, s, wq);
    hipLaunchKernelGGL(weight_quantize_kernel, dim3((unsigned)blocks), dim3(HQ_THREADS), 0, s, Wf, n, wq, Wq);
    return launch_status();
}

int hq_probe_mfma_rate(int32_t blocks, int32_t iters, int32_t *sink, void *stream)
{
    if (!sink || blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 20)) return HQ_E_BADARG;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(HQ_THREADS), 0, as_stream(stream), iters, sink);
    return launch_status();
}

} // extern "C"
