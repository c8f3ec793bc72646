// Device-side helpers shared by the HIP kernels of the hq library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include "../../include/hq.h"

typedef int v4i  __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define HQ_THREADS 256                     // every compute kernel runs 4 wavefronts of 64 lanes

// x / d by multiplication, for d >= 1 and x * d < 2^32: magic = (unsigned)ceil(2^32 / d), which for
// d == 1 wraps to 0 and is then taken as "no division".  The host computes the constant.
__host__ __device__ inline unsigned hq_magic32(unsigned d) { return (unsigned)(((1ull << 32) + d - 1) / d); }
__device__ inline unsigned hq_magic_div(unsigned x, unsigned magic) { return magic ? __umulhi(x, magic) : x; }

// ---------------------------------------------------------------------------------------
// 3-byte pixels (RGB inputs): a lane's 4-byte word of the reduction starts at any byte address and
// can hold bytes of two taps.  Words are loaded unaligned and the unwanted bytes replaced under a
// byte mask.
// ---------------------------------------------------------------------------------------

// Bytes e of a 32-bit word with lo <= e < hi (little endian), as a mask of whole bytes.
__device__ inline unsigned hq_bytemask(int lo, int hi)
{
    lo = max(lo, 0); hi = min(hi, 4);
    if (hi <= lo) return 0u;
    const unsigned upto_hi = hi == 4 ? 0xffffffffu : (1u << (8 * hi)) - 1u;
    return upto_hi & ~((1u << (8 * lo)) - 1u);
}

// 16 consecutive bytes starting at p (any alignment) of a tensor that occupies [begin, end): aligned loads
// of the five 32-bit words that hold them (one 16-byte and one 4-byte load where all five lie inside the
// tensor, guarded single words at its first and last bytes), then a byte-wise funnel shift.  Unaligned
// word loads are served far more slowly.  Bytes outside the tensor arrive as anything: the caller masks them
// (they belong to taps outside the image).  An aligned word that holds the tensor's last byte is read
// whole, i.e. up to the next multiple of 4 of `end`.
__device__ inline v4i hq_load16_any(const int8_t *p, const int8_t *begin, const int8_t *end)
{
    // (pointer arithmetic only: a pointer rebuilt from an integer would lose its address space and every load
    // below would become a flat load, which the compiler can only wait for all at once)
    const unsigned sh = (unsigned)(reinterpret_cast<uintptr_t>(p) & 3);
    const int8_t *a = p - sh;
    const int8_t *end4 = end + ((4u - (unsigned)(reinterpret_cast<uintptr_t>(end) & 3)) & 3u);
    int w[5];
    // one uniform branch: wavefronts that touch neither end of the tensor (all but a few) take the two wide
    // loads; the others load word by word from addresses moved inside the tensor where they would fall outside
    const bool inner = a >= begin && a + 20 <= end4;
    if (__builtin_amdgcn_ballot_w64(!inner) == 0) {
        v4i x;
        __builtin_memcpy(&x, __builtin_assume_aligned(a, 4), 16);
        w[0] = x[0]; w[1] = x[1]; w[2] = x[2]; w[3] = x[3];
        w[4] = *reinterpret_cast<const int *>(a + 16);
    } else {
        const int8_t *safe = begin + ((4u - (unsigned)(reinterpret_cast<uintptr_t>(begin) & 3)) & 3u);
#pragma unroll
        for (int d = 0; d < 5; d++) {
            const int8_t *q = a + 4 * d;
            const bool in = q >= begin && q < end4;
            const int x = *reinterpret_cast<const int *>(in ? q : safe);
            w[d] = in ? x : 0;
        }
    }
    v4i v;
#pragma unroll
    for (int d = 0; d < 4; d++) v[d] = (int)__builtin_amdgcn_alignbyte((unsigned)w[d + 1], (unsigned)w[d], sh);
    return v;
}

// ---------------------------------------------------------------------------------------
// Quantizer arithmetic.  Each fp32 operation rounds once (no contraction), so that the
// result is a function of the operands alone.
// ---------------------------------------------------------------------------------------

// Quantizer of a range (qmin, qmax): asymmetric grids are widened to contain real zero.
__device__ inline hq_qparams hq_qparams_from_range(float qmin, float qmax, int symmetric, int qlo, int qhi)
{
    hq_qparams q;
    if (symmetric) {
        float amax = fmaxf(fabsf(qmin), fabsf(qmax));
        q.scale = amax > 0.0f ? __fdiv_rn(amax, (float)qhi) : 1.0f;
        q.zero_point = 0;
        return q;
    }
    float lo = fminf(qmin, 0.0f), hi = fmaxf(qmax, 0.0f);
    float width = __fsub_rn(hi, lo);
    float s = width > 0.0f ? __fdiv_rn(width, (float)(qhi - qlo)) : 1.0f;
    float z = rintf(__fsub_rn((float)qlo, __fdiv_rn(lo, s)));
    z = fminf(fmaxf(z, (float)qlo), (float)qhi);
    q.scale = s;
    q.zero_point = (int)z;
    return q;
}

// Order-preserving map between fp32 values and signed 32-bit keys (its own inverse on the bit
// pattern): integer min / max and their atomics then order real values.  Used by the statistics
// of real-valued tensors; -0 is made +0 first so that equal values have equal keys.
__device__ inline int hq_float_key(float x)
{
    const int b = __float_as_int(x + 0.0f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ inline float hq_key_float(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

// ---------------------------------------------------------------------------------------
// eq. (2)-(3): q <- (1 - eta) * g + eta * q, each product and the sum rounded once.
// ---------------------------------------------------------------------------------------
__device__ inline void hq_ema_update(hq_range *r, float gmin, float gmax)
{
    if (!r->initialized) {
        r->qmin = gmin; r->qmax = gmax; r->initialized = 1;
    } else {
        const float w = __fsub_rn(1.0f, r->eta);
        r->qmin = __fadd_rn(__fmul_rn(w, gmin), __fmul_rn(r->eta, r->qmin));
        r->qmax = __fadd_rn(__fmul_rn(w, gmax), __fmul_rn(r->eta, r->qmax));
    }
    r->qp = hq_qparams_from_range(r->qmin, r->qmax, r->symmetric, r->qlo, r->qhi);
}

// ---------------------------------------------------------------------------------------
// Saturation-driven update (Sec. 4 names the saturation ratio as a statistic; the rule is this
// library's, stated with hq_range_update_saturation).
// ---------------------------------------------------------------------------------------

// ln x for a positive normal x by a fixed sequence of fp32 operations, each rounded once:
// x = m * 2^e, m in [sqrt(1/2), sqrt(2)), s = (m - 1) / (m + 1), ln x = e ln 2 + 2 s (1 + s^2/3 + s^4/5 + s^6/7).
__device__ inline float hq_ln_fixed(float x)
{
    const unsigned bits = __float_as_uint(x);
    int e = (int)((bits >> 23) & 0xffu) - 127;
    float m = __uint_as_float((bits & 0x007fffffu) | 0x3f800000u);
    if (m > 1.41421354f) { m = __fmul_rn(m, 0.5f); e += 1; }
    const float sq = __fdiv_rn(__fsub_rn(m, 1.0f), __fadd_rn(m, 1.0f));
    const float s2 = __fmul_rn(sq, sq);
    float p = __fmul_rn(s2, 1.0f / 7.0f);
    p = __fadd_rn(p, 0.2f);
    p = __fmul_rn(p, s2);
    p = __fadd_rn(p, 1.0f / 3.0f);
    p = __fmul_rn(p, s2);
    p = __fadd_rn(p, 1.0f);
    const float lm = __fmul_rn(__fmul_rn(2.0f, sq), p);
    return __fadd_rn(__fmul_rn((float)e, 0.693147182f), lm);
}

__device__ inline void hq_saturation_update(hq_range *r, hq_saturation *sat, unsigned long long clipped,
                                            unsigned long long count, float gmin, float gmax)
{
    if (!r->initialized) {
        r->qmin = gmin; r->qmax = gmax; r->initialized = 1;
        sat->streak = 0;
    } else {
        const float alpha = __fdiv_rn((float)clipped, (float)count);
        if (alpha >= sat->alpha_min && alpha <= sat->alpha_max) {
            sat->streak = 0;
        } else {
            sat->streak += 1;
            if (sat->streak > sat->tau) {
                const float fl = __fdiv_rn(0.5f, (float)count);
                const float ah = fminf(fmaxf(alpha, fl), 0.5f);
                const float rho = __fdiv_rn(hq_ln_fixed(sat->alpha_target), hq_ln_fixed(ah));
                r->qmin = __fmul_rn(rho, r->qmin);
                r->qmax = __fmul_rn(rho, r->qmax);
                sat->streak = 0;
            }
        }
    }
    r->qp = hq_qparams_from_range(r->qmin, r->qmax, r->symmetric, r->qlo, r->qhi);
}

// Everything the epilogue needs to turn a zero-point-corrected accumulator into a code.
struct HqRequant {
    float mult;        // (s_a * s_b) / s_out
    float flo, fhi;    // grid bounds relative to the zero point, as floats
    int   z;
};

__device__ inline HqRequant hq_make_requant(float acc_scale, hq_qparams out, int qlo, int qhi)
{
    HqRequant r;
    r.mult = __fdiv_rn(acc_scale, out.scale);
    r.flo = (float)(qlo - out.zero_point);
    r.fhi = (float)(qhi - out.zero_point);
    r.z = out.zero_point;
    return r;
}

// One fp32 multiply, round half to even, clamp in float, then the zero point.
__device__ inline int hq_requant(int c, const HqRequant &q, unsigned &nlo, unsigned &nhi)
{
    float r = rintf(__fmul_rn((float)c, q.mult));
    nlo += (r < q.flo) ? 1u : 0u;
    nhi += (r > q.fhi) ? 1u : 0u;
    r = fminf(fmaxf(r, q.flo), q.fhi);
    return (int)r + q.z;
}

// ---------------------------------------------------------------------------------------
// Fused epilogue of the MFMA kernels: a lane's zero-point-corrected accumulators -> codes,
// with min / max and exact clip counts folded in (Sec. 4, steps 1 and 2).
// Per value: convert, multiply, round (the requantization of the static quantizer), add the
// zero point, pack.  Clipped values are counted per lane from the rounded floats, and only in
// groups whose extreme accumulators clip: requantization is monotone in the accumulator, so
// the extremes decide for the whole group.
// ---------------------------------------------------------------------------------------
struct HqEpilogue {
    float mult;          // (s_a * s_b) / s_out
    float flo, fhi;      // grid bounds relative to the zero point
    float zoff;          // zero point + 128: codes are formed as unsigned bytes, see below
    bool full_grid;      // grid is -128..127: the saturating pack is the whole clamp
};

__device__ inline HqEpilogue hq_make_epilogue(float acc_scale, const hq_range *r)
{
    HqEpilogue e;
    e.mult = __fdiv_rn(acc_scale, r->qp.scale);
    e.flo = (float)(r->qlo - r->qp.zero_point);
    e.fhi = (float)(r->qhi - r->qp.zero_point);
    e.zoff = (float)(r->qp.zero_point + 128);
    e.full_grid = r->qlo == -128 && r->qhi == 127;
    return e;
}

__device__ inline float hq_round_scaled(int c, float mult) { return rintf(__fmul_rn((float)c, mult)); }

// 16 bytes per lane from global memory straight into LDS (global_load_lds_dwordx4): lane l of the wavefront
// lands at wave_base + 16 * l.  Written as an asm statement because the compiler, once it has issued such a load
// itself, waits for every outstanding LDS read before using any of them (it stops counting them), which
// defeats fragment double buffering in the loops that follow.  The caller waits for the load with an explicit
// "s_waitcnt vmcnt(..)" before a barrier; the compiler's own counts stay safe because loads retire in order.
__device__ inline void hq_global_to_lds16(const void *src, void *wave_base)
{
    const unsigned m = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) void *)wave_base);
    unsigned keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "v"(src), "s"(m) : "memory");
}

// Three-operand integer minimum / maximum (v_min3_i32 / v_max3_i32).  Written out because the compiler
// balances a chain of two-operand minima into a tree and then needs 12 instructions for 16 values, not 8.
__device__ inline int hq_min3(int a, int b, int c)
{
    int r;
    asm("v_min3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ inline int hq_max3(int a, int b, int c)
{
    int r;
    asm("v_max3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// N = 4 or 16 accumulators -> N / 4 words of signed codes.  v_cvt_pk_u8_f32 saturates to
// 0..255, which after the flip of the top bits is the clamp to -128..127.
template <int N, bool FULL_GRID>
__device__ inline void hq_requant_group(const int *c, const HqEpilogue &ep, int &mn, int &mx,
                                        unsigned &w_lo, unsigned &w_hi, int *words)
{
    int gmn = c[0], gmx = c[0];
#pragma unroll
    for (int e = 1; e + 1 < N; e += 2) { gmn = hq_min3(gmn, c[e], c[e + 1]); gmx = hq_max3(gmx, c[e], c[e + 1]); }
    gmn = min(gmn, c[N - 1]); gmx = max(gmx, c[N - 1]);
    mn = min(mn, gmn); mx = max(mx, gmx);
    float f[N];
#pragma unroll
    for (int e = 0; e < N; e++) f[e] = hq_round_scaled(c[e], ep.mult);
    if (__any(hq_round_scaled(gmx, ep.mult) > ep.fhi || hq_round_scaled(gmn, ep.mult) < ep.flo)) {
        // rounded values and bounds are whole numbers: clamping the difference to [0, 1] is the
        // indicator of a clipped value (a subtraction with the clamp modifier, no compare)
        float nh = 0.0f, nl = 0.0f;
#pragma unroll
        for (int e = 0; e < N; e++) {
            nh += __builtin_amdgcn_fmed3f(f[e] - ep.fhi, 0.0f, 1.0f);
            nl += __builtin_amdgcn_fmed3f(ep.flo - f[e], 0.0f, 1.0f);
        }
        w_hi += (unsigned)nh; w_lo += (unsigned)nl;
    }
#pragma unroll
    for (int g = 0; g < N / 4; g++) {
        unsigned w = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            float v = f[4 * g + e];
            if (!FULL_GRID) v = __builtin_amdgcn_fmed3f(v, ep.flo, ep.fhi);
            w = __builtin_amdgcn_cvt_pk_u8_f32(v + ep.zoff, e, w);
        }
        words[g] = (int)(w ^ 0x80808080u);
    }
}

// ---------------------------------------------------------------------------------------
// Stochastic rounding (the paper quantizes gradients with it, Sec. 5 experimental setup, after
// Gupta et al. 2015): the scaled accumulator x rounds up with probability x - floor(x).  Each
// output element draws its 24 random bits from a counter-based generator keyed on the element's
// linear index in its tensor and a 64-bit seed, so the result does not depend on how the launch
// is tiled.  The generator: the low index word through the finalizer of MurmurHash3, with the
// first key word added and the high index word (times an odd constant) plus the second key
// word folded in between its two rounds, closed by a multiply with the golden-ratio constant
// and a xor-shift.
// ---------------------------------------------------------------------------------------
struct HqSr { unsigned k0, k1; };          // low and high half of the seed

__device__ inline unsigned hq_sr_bits(unsigned idx_lo, unsigned hi_term, unsigned k0)
{
    unsigned h = idx_lo;                   // hi_term = idx_hi * 0x85ebca77 + k1
    h ^= h >> 16; h *= 0x85ebca6bu; h += k0;
    h ^= hi_term;
    h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    h *= 0x9e3779b1u; h ^= h >> 15;
    return h;
}

// One value (the depthwise stencil's epilogue): as hq_requant, with stochastic rounding.
__device__ inline int hq_requant_sr(int c, const HqRequant &q, const HqSr &sr, size_t idx, unsigned &nlo, unsigned &nhi)
{
    const unsigned bits = hq_sr_bits((unsigned)idx, (unsigned)(idx >> 32) * 0x85ebca77u + sr.k1, sr.k0);
    const float x = __fmul_rn((float)c, q.mult), fl = floorf(x);
    const float u = __fmul_rn((float)(bits >> 8), 1.0f / 16777216.0f);
    float r = __fsub_rn(x, fl) > u ? __fadd_rn(fl, 1.0f) : fl;
    nlo += (r < q.flo) ? 1u : 0u;
    nhi += (r > q.fhi) ? 1u : 0u;
    r = fminf(fmaxf(r, q.flo), q.fhi);
    return (int)r + q.z;
}

// As hq_requant_group, with stochastic rounding; idx0 is the tensor index of c[0], the N values
// are consecutive elements.
template <int N, bool FULL_GRID>
__device__ inline void hq_requant_group_sr(const int *c, const HqEpilogue &ep, const HqSr &sr, size_t idx0, int &mn,
                                           int &mx, unsigned &w_lo, unsigned &w_hi, int *words)
{
    int gmn = c[0], gmx = c[0];
#pragma unroll
    for (int e = 1; e + 1 < N; e += 2) { gmn = hq_min3(gmn, c[e], c[e + 1]); gmx = hq_max3(gmx, c[e], c[e + 1]); }
    gmn = min(gmn, c[N - 1]); gmx = max(gmx, c[N - 1]);
    mn = min(mn, gmn); mx = max(mx, gmx);
    const unsigned lo0 = (unsigned)idx0, hi0 = (unsigned)(idx0 >> 32);
    const unsigned term0 = hi0 * 0x85ebca77u + sr.k1, term1 = (hi0 + 1u) * 0x85ebca77u + sr.k1;
    float f[N];
#pragma unroll
    for (int e = 0; e < N; e++) {
        const unsigned lo = lo0 + (unsigned)e;
        const unsigned bits = hq_sr_bits(lo, lo < lo0 ? term1 : term0, sr.k0);       // carry into the high word
        const float x = __fmul_rn((float)c[e], ep.mult), fl = floorf(x);
        const float u = __fmul_rn((float)(bits >> 8), 1.0f / 16777216.0f);
        f[e] = __fsub_rn(x, fl) > u ? __fadd_rn(fl, 1.0f) : fl;
    }
    // the rounded value lies in [floor(x), floor(x) + 1]: the group's extremes decide whether any can clip
    if (__any(__fadd_rn(floorf(__fmul_rn((float)gmx, ep.mult)), 1.0f) > ep.fhi || floorf(__fmul_rn((float)gmn, ep.mult)) < ep.flo)) {
        float nh = 0.0f, nl = 0.0f;
#pragma unroll
        for (int e = 0; e < N; e++) {
            nh += __builtin_amdgcn_fmed3f(f[e] - ep.fhi, 0.0f, 1.0f);
            nl += __builtin_amdgcn_fmed3f(ep.flo - f[e], 0.0f, 1.0f);
        }
        w_hi += (unsigned)nh; w_lo += (unsigned)nl;
    }
#pragma unroll
    for (int g = 0; g < N / 4; g++) {
        unsigned w = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            float v = f[4 * g + e];
            if (!FULL_GRID) v = __builtin_amdgcn_fmed3f(v, ep.flo, ep.fhi);
            w = __builtin_amdgcn_cvt_pk_u8_f32(v + ep.zoff, e, w);
        }
        words[g] = (int)(w ^ 0x80808080u);
    }
}

// min / max alone (pass 1 of the dynamic baseline keeps the 32-bit values)
template <int N> __device__ inline void hq_minmax_group(const int *c, int &mn, int &mx)
{
#pragma unroll
    for (int e = 0; e + 1 < N; e += 2) { mn = hq_min3(mn, c[e], c[e + 1]); mx = hq_max3(mx, c[e], c[e + 1]); }
}

__device__ inline unsigned hq_pack4(int a, int b, int c, int d)
{
    return (unsigned)(a & 0xff) | ((unsigned)(b & 0xff) << 8) | ((unsigned)(c & 0xff) << 16) | ((unsigned)d << 24);
}

// ---------------------------------------------------------------------------------------
// Wavefront and workgroup reductions for the online statistics.
// ---------------------------------------------------------------------------------------

// Exchange with the lane whose index differs in bit `k` (k < 32: ds_swizzle inside each
// half of the wavefront; k == 32: across the halves).
template <int K> __device__ inline int hq_lane_xor(int v)
{
    if (K < 32) return __builtin_amdgcn_ds_swizzle(v, (K << 10) | 0x1f);
    return __shfl_xor(v, 32);
}

template <typename Op> __device__ inline int hq_wave_reduce(int v, Op op)
{
    v = op(v, hq_lane_xor<1>(v));
    v = op(v, hq_lane_xor<2>(v));
    v = op(v, hq_lane_xor<4>(v));
    v = op(v, hq_lane_xor<8>(v));
    v = op(v, hq_lane_xor<16>(v));
    v = op(v, hq_lane_xor<32>(v));
    return v;
}

struct HqMin { __device__ int operator()(int a, int b) const { return a < b ? a : b; } };
struct HqMax { __device__ int operator()(int a, int b) const { return a > b ? a : b; } };
struct HqAdd { __device__ int operator()(int a, int b) const { return a + b; } };

// Merges one workgroup's statistics into the tensor's record: wavefront reduction, a
// second level through LDS, then one atomic per field from one lane, into the partial record
// chosen by the workgroup's index: consecutive workgroups land on different 128-byte lines, so
// a launch's atomics do not queue on one address.  `red` is LDS space for 4 * (NTHREADS / 64)
// ints.  Must be called by all NTHREADS threads of the workgroup.
template <int NTHREADS>
__device__ inline void hq_block_stats_commit_n(int mn, int mx, unsigned nlo, unsigned nhi,
                                               hq_stats *st, int *red)
{
    mn = hq_wave_reduce(mn, HqMin());
    mx = hq_wave_reduce(mx, HqMax());
    nlo = (unsigned)hq_wave_reduce((int)nlo, HqAdd());
    nhi = (unsigned)hq_wave_reduce((int)nhi, HqAdd());
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    constexpr int NW = NTHREADS / 64;
    if (lane == 0) { red[wave] = mn; red[NW + wave] = mx; red[2 * NW + wave] = (int)nlo; red[3 * NW + wave] = (int)nhi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long lo = 0, hi = 0;
        for (int w = 0; w < NW; w++) {
            mn = min(mn, red[w]); mx = max(mx, red[NW + w]);
            lo += (unsigned)red[2 * NW + w]; hi += (unsigned)red[3 * NW + w];
        }
        const unsigned block = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        hq_stats_part *part = &st->part[block % HQ_STATS_PARTS];
        if (mn <= mx) { atomicMin(&part->acc_min, mn); atomicMax(&part->acc_max, mx); }
        if (lo) atomicAdd((unsigned long long *)&part->clip_lo, lo);
        if (hi) atomicAdd((unsigned long long *)&part->clip_hi, hi);
    }
}

__device__ inline void hq_block_stats_commit(int mn, int mx, unsigned nlo, unsigned nhi, hq_stats *st, int *red)
{
    hq_block_stats_commit_n<HQ_THREADS>(mn, mx, nlo, nhi, st, red);
}

// Moves what the partial records hold into the record's leading fields and empties them.
// One wavefront (HQ_STATS_PARTS == 64 lanes, lane = partial record), registers only.  Lane 0
// writes the leading fields; every lane returns their new values.
struct HqStatsFolded { int acc_min, acc_max; unsigned long long clip_lo, clip_hi; };

__device__ inline unsigned long long hq_wave_sum64(unsigned long long v)
{
#pragma unroll
    for (int k = 1; k < 64; k <<= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, k), hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), k);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

__device__ inline HqStatsFolded hq_stats_fold_wave(hq_stats *st)
{
    static_assert(HQ_STATS_PARTS == 64, "one lane per partial record");
    const int lane = threadIdx.x & 63;
    hq_stats_part *p = &st->part[lane];
    const int pmn = p->acc_min, pmx = p->acc_max;
    const unsigned long long plo = p->clip_lo, phi = p->clip_hi;
    HqStatsFolded f;
    f.acc_min = st->acc_min; f.acc_max = st->acc_max; f.clip_lo = st->clip_lo; f.clip_hi = st->clip_hi;
    p->acc_min = INT_MAX; p->acc_max = INT_MIN; p->clip_lo = 0; p->clip_hi = 0;
    f.acc_min = min(f.acc_min, hq_wave_reduce(pmn, HqMin()));
    f.acc_max = max(f.acc_max, hq_wave_reduce(pmx, HqMax()));
    f.clip_lo += hq_wave_sum64(plo);
    f.clip_hi += hq_wave_sum64(phi);
    if (lane == 0) { st->acc_min = f.acc_min; st->acc_max = f.acc_max; st->clip_lo = f.clip_lo; st->clip_hi = f.clip_hi; }
    return f;
}

// eq. (2)-(3) for one quantizer, by one wavefront: folds the statistics record, moves the range,
// derives the quantizer, empties the record.  With count == 0 the range is left as it is.
__device__ inline void hq_range_update_wave(hq_range *r, hq_stats *st)
{
    // every load is issued before anything waits: one memory round trip
    hq_range rr = *r;
    const float acc_scale = st->acc_scale;
    const unsigned fp32_keys = st->fp32_keys;
    const unsigned long long count = st->count;
    const HqStatsFolded f = hq_stats_fold_wave(st);
    if ((threadIdx.x & 63) == 0) {
        if (count != 0) {
            if (fp32_keys) hq_ema_update(&rr, hq_key_float(f.acc_min), hq_key_float(f.acc_max));
            else hq_ema_update(&rr, __fmul_rn(acc_scale, (float)f.acc_min), __fmul_rn(acc_scale, (float)f.acc_max));
            *r = rr;
        }
        st->acc_min = INT_MAX; st->acc_max = INT_MIN; st->acc_scale = 0.0f; st->fp32_keys = 0;
        st->clip_lo = 0; st->clip_hi = 0; st->count = 0;           // the partial records are already empty
    }
}

// Range updates that ride along with another launch: the workgroups past `first` of that launch
// (one per quantizer, their first wavefront) run eq. (2)-(3) instead of the launch's own work.
struct HqRideAlong { hq_range *r; hq_stats *st; int n; int first; };

__device__ inline bool hq_ride_along(const HqRideAlong &ra)
{
    if (ra.n == 0 || (int)blockIdx.x < ra.first) return false;
    if (threadIdx.x < 64) hq_range_update_wave(ra.r + (blockIdx.x - ra.first), ra.st + (blockIdx.x - ra.first));
    return true;
}
