// Element-wise quantizers for FP32 tensors that are produced outside the GEMMs (normalisation or
// activation outputs): the in-hindsight quantizer (Sec. 3.2 static quantization with the range of
// eq. (2)-(3); one pass: 4 bytes in, 1 byte out per element, statistics gathered on the way) and its
// dynamic counterpart (eq. (1): a min/max pass over the tensor, then the quantizing pass: 8 bytes in,
// 1 byte out).  Both are bound by HBM; the arithmetic per element is a multiply, a round, a clamp.
#include "hq_device.h"
#include "hq_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TQ_GROUP = 16;        // elements per thread and trip: four 16-byte loads, one 16-byte store

// QUANT: write codes and count the clipped ones; MINMAX: gather the tensor's minimum and maximum
// as order-preserving keys.  The in-hindsight pass does both, the dynamic passes one each.
// SR: stochastic rounding, the draw keyed on the element's index in the tensor and the seed.
template <bool QUANT, bool MINMAX, bool SR>
__global__ __launch_bounds__(HQ_THREADS) void tensor_pass_kernel(const float *__restrict__ x, size_t n,
                                                                 const hq_range *r, const hq_qparams *qp,
                                                                 int8_t *__restrict__ out, hq_qparams *q_out,
                                                                 hq_stats *st, HqSr sr)
{
    __shared__ int red[4 * (HQ_THREADS / 64)];
    HqRequant rq = {};
    if (QUANT) rq = hq_make_requant(1.0f, *qp, r->qlo, r->qhi);       // a real value is an accumulator of unit 1
    int mn = INT_MAX, mx = INT_MIN;
    unsigned nlo = 0, nhi = 0;
    auto one = [&](float v, size_t idx) __attribute__((always_inline)) -> int {
        if (MINMAX) { const int k = hq_float_key(v); mn = min(mn, k); mx = max(mx, k); }
        if (!QUANT) return 0;
        float q;
        if (SR) {
            const unsigned bits = hq_sr_bits((unsigned)idx, (unsigned)(idx >> 32) * 0x85ebca77u + sr.k1, sr.k0);
            const float y = __fmul_rn(v, rq.mult), fl = floorf(y);
            const float u = __fmul_rn((float)(bits >> 8), 1.0f / 16777216.0f);
            q = __fsub_rn(y, fl) > u ? __fadd_rn(fl, 1.0f) : fl;
        } else {
            q = rintf(__fmul_rn(v, rq.mult));
        }
        nlo += (q < rq.flo) ? 1u : 0u;
        nhi += (q > rq.fhi) ? 1u : 0u;
        q = fminf(fmaxf(q, rq.flo), rq.fhi);
        return (int)q + rq.z;
    };
    const size_t groups = n / TQ_GROUP, step = (size_t)gridDim.x * blockDim.x;
    for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += step) {
        const v4f *src = reinterpret_cast<const v4f *>(x) + 4 * g;
        v4f v[4];
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = src[k];
        v4i packed;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const size_t i0 = g * TQ_GROUP + 4 * k;
            const int c0 = one(v[k][0], i0), c1 = one(v[k][1], i0 + 1), c2 = one(v[k][2], i0 + 2), c3 = one(v[k][3], i0 + 3);
            packed[k] = (int)hq_pack4(c0, c1, c2, c3);
        }
        if (QUANT) reinterpret_cast<v4i *>(out)[g] = packed;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (size_t i = groups * TQ_GROUP; i < n; i++) {               // fewer than 16 elements
            const int c = one(x[i], i);
            if (QUANT) out[i] = (int8_t)c;
        }
        if (MINMAX) {
            atomicAdd((unsigned long long *)&st->count, (unsigned long long)n);
            st->acc_scale = 1.0f;
            st->fp32_keys = 1;
        }
        if (QUANT && q_out != qp) *q_out = *qp;
    }
    hq_block_stats_commit(mn, mx, nlo, nhi, st, red);
}

// Dynamic quantizer, between the passes: the quantizer of the tensor just scanned.
__global__ __launch_bounds__(64) void tensor_mid_kernel(int mode, hq_range *r, hq_stats *st, hq_qparams *q_out)
{
    const unsigned long long count = st->count;
    const HqStatsFolded f = hq_stats_fold_wave(st);
    if (threadIdx.x != 0) return;
    if (count == 0) { *q_out = r->qp; return; }                        // empty tensor: nothing to estimate from
    const float gmin = hq_key_float(f.acc_min), gmax = hq_key_float(f.acc_max);
    if (mode == HQ_DYN_RUNNING) {
        hq_ema_update(r, gmin, gmax);
        *q_out = r->qp;
    } else {
        if (!r->initialized) hq_ema_update(r, gmin, gmax);
        *q_out = hq_qparams_from_range(gmin, gmax, r->symmetric, r->qlo, r->qhi);
    }
}

inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? HQ_OK : HQ_E_HIP; }

inline unsigned pass_blocks(size_t n)
{
    size_t blocks = (n / TQ_GROUP + HQ_THREADS - 1) / HQ_THREADS;
    if (blocks < 1) blocks = 1;
    if (blocks > 256u * 8u) blocks = 256u * 8u;                        // grid-stride beyond eight workgroups per CU
    return (unsigned)blocks;
}

} // namespace

extern "C" {

int hq_tensor_quantize(const float *X, size_t n, const hq_range *r, int8_t *Q, hq_qparams *q_out,
                       hq_stats *st, void *stream)
{
    if (!r || !q_out || !st || (n && (!X || !Q))) return HQ_E_BADARG;
    if (misaligned(X, 16) || misaligned(Q, 16) || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL((tensor_pass_kernel<true, true, false>), dim3(pass_blocks(n)), dim3(HQ_THREADS), 0,
                       reinterpret_cast<hipStream_t>(stream), X, n, r, &r->qp, Q, q_out, st, HqSr{0, 0});
    return launch_status();
}

int hq_tensor_quantize_sr(const float *X, size_t n, const hq_range *r, uint64_t seed, int8_t *Q,
                          hq_qparams *q_out, hq_stats *st, void *stream)
{
    if (!r || !q_out || !st || (n && (!X || !Q))) return HQ_E_BADARG;
    if (misaligned(X, 16) || misaligned(Q, 16) || misaligned(st, 128)) return HQ_E_BADARG;
    hipLaunchKernelGGL((tensor_pass_kernel<true, true, true>), dim3(pass_blocks(n)), dim3(HQ_THREADS), 0,
                       reinterpret_cast<hipStream_t>(stream), X, n, r, &r->qp, Q, q_out, st,
                       HqSr{(unsigned)seed, (unsigned)(seed >> 32)});
    return launch_status();
}

int hq_tensor_quantize_dynamic(int32_t mode, const float *X, size_t n, hq_range *r, int8_t *Q,
                               hq_qparams *q_out, hq_stats *st, void *stream)
{
    if (mode != HQ_DYN_CURRENT && mode != HQ_DYN_RUNNING) return HQ_E_BADARG;
    if (!r || !q_out || !st || (n && (!X || !Q))) return HQ_E_BADARG;
    if (misaligned(X, 16) || misaligned(Q, 16) || misaligned(st, 128)) return HQ_E_BADARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const unsigned blocks = pass_blocks(n);
    hipLaunchKernelGGL((tensor_pass_kernel<false, true, false>), dim3(blocks), dim3(HQ_THREADS), 0, s, X, n, r,
                       (const hq_qparams *)nullptr, (int8_t *)nullptr, (hq_qparams *)nullptr, st, HqSr{0, 0});
    hipLaunchKernelGGL(tensor_mid_kernel, dim3(1), dim3(64), 0, s, (int)mode, r, st, q_out);
    hipLaunchKernelGGL((tensor_pass_kernel<true, false, false>), dim3(blocks), dim3(HQ_THREADS), 0, s, X, n, r,
                       (const hq_qparams *)q_out, Q, q_out, st, HqSr{0, 0});
    return launch_status();
}

} // extern "C"
