/*
 * hq_oracle.c -- CPU oracle for the in-hindsight quantized-training layer path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the GPU library and must never be reached from the product path; only
 * tests, the smoke check and the CPU-baseline leg of the benchmark load it.
 *
 * What it computes (paper: "In-Hindsight Quantization Range Estimation for
 * Quantized Training", arXiv 2105.04246):
 *   - the three linear operations of a quantized layer (Sec. 3.1, Fig. 1):
 *     forward Y = X~ W~, input gradient G_X = G~_Y W~^T, weight gradient
 *     G_W = X~^T G~_Y, on 8-bit codes with a wide integer accumulator
 *     (Sec. 3.2: accumulator output is 32 bit);
 *   - the min-max statistics of the accumulator output, eq. (1);
 *   - static quantization of the accumulator output with a range known in
 *     advance (Sec. 3.2), and dynamic quantization with the current range;
 *   - the in-hindsight min-max range update, eq. (2)-(3), and its t=0
 *     initialisation (Sec. 4.1);
 *   - the saturation ratio counters (Sec. 4, footnote).
 *
 * The paper never writes the uniform quantizer out; the formulas used here are
 * the readings listed in the design notes of this repository (asymmetric:
 * range widened to contain 0, scale = width / (qhi-qlo), zero point rounded
 * half-to-even and clamped; symmetric: scale = max|.| / qhi, zero point 0).
 *
 * Parity pins: every function below is pinned by tests that do not call it to
 * produce their expectation (brute force in pure Python integers, NumPy int64
 * matmul on an explicit im2col matrix, adjoint identities, closed forms of the
 * EMA recursion, exhaustive integer round-half-even, values of Table 5 for
 * the traffic model which lives in traffic.py).  Nothing here is unpinned.
 *
 * Conventions.  Tensors are NHWC / row-major.  Codes are signed 8-bit; an
 * unsigned grid 0..255 is stored shifted by -128 and its zero point with it.
 * A real value is scale * (code - zero_point).  Out-of-image taps of a
 * convolution hold real zero, i.e. they contribute nothing to any sum.
 * Weights: conv/linear [Cout][R][S][C]; depthwise [R][S][C].
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <limits.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t kind;            /* 0 linear, 1 conv2d, 2 depthwise conv2d            */
    int32_t B, H, W, C;      /* input NHWC; linear: B rows, C = reduction length  */
    int32_t R, S, stride, pad;
    int32_t Cout;            /* output channels (depthwise: == C)                  */
} hqo_problem;

typedef struct {
    float   qmin, qmax;      /* eq. (2)-(3) state, real units                      */
    float   eta;             /* momentum                                           */
    int32_t qlo, qhi;        /* integer grid                                       */
    int32_t symmetric;
    int32_t initialized;     /* 0 until q^0 has been set from the first batch      */
    float   scale;           /* quantizer derived from (qmin,qmax)                 */
    int32_t zero_point;
} hqo_range;

int hqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

void hqo_out_hw(const hqo_problem *p, int32_t *OH, int32_t *OW)
{
    *OH = out_dim(p->H, p->R, p->stride, p->pad);
    *OW = out_dim(p->W, p->S, p->stride, p->pad);
}

/* ------------------------------------------------------------------------- */
/* Linear operations on codes, zero points removed, exact integers.           */
/* Return value: 0 ok, 1 if some result does not fit a 32-bit accumulator     */
/* (Sec. 3.2 assumes it does).                                                */
/* ------------------------------------------------------------------------- */

/* One forward output row (all output channels of one output pixel).          */
static int fwd_row(const hqo_problem *p, const int8_t *X, int zx, const int8_t *Wt,
                   int64_t m, int32_t *out)
{
    int OH, OW; hqo_out_hw(p, &OH, &OW);
    int ow = (int)(m % OW), oh = (int)((m / OW) % OH), b = (int)(m / ((int64_t)OW * OH));
    int bad = 0;
    for (int n = 0; n < p->Cout; n++) {
        int64_t sum = 0;
        for (int r = 0; r < p->R; r++) {
            int ih = oh * p->stride - p->pad + r;
            if (ih < 0 || ih >= p->H) continue;
            for (int s = 0; s < p->S; s++) {
                int iw = ow * p->stride - p->pad + s;
                if (iw < 0 || iw >= p->W) continue;
                const int8_t *x = X + (((int64_t)b * p->H + ih) * p->W + iw) * p->C;
                if (p->kind == 2) {
                    sum += (int64_t)((int)x[n] - zx) * Wt[((int64_t)r * p->S + s) * p->C + n];
                } else {
                    const int8_t *w = Wt + (((int64_t)n * p->R + r) * p->S + s) * p->C;
                    for (int c = 0; c < p->C; c++) sum += (int64_t)((int)x[c] - zx) * w[c];
                }
            }
        }
        if (sum > INT32_MAX || sum < INT32_MIN) bad = 1;
        out[n] = (int32_t)sum;
    }
    return bad;
}

/* Forward, Sec. 3.1: c[m,n] = sum over taps and channels of (X~ - z_x) W~.   */
int hqo_fwd(const hqo_problem *p, const int8_t *X, int zx, const int8_t *Wt, int32_t *c)
{
    int OH, OW; hqo_out_hw(p, &OH, &OW);
    int64_t M = (int64_t)p->B * OH * OW;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; m++) bad |= fwd_row(p, X, zx, Wt, m, c + m * p->Cout);
    return bad;
}

/* Same, for a caller-chosen list of output pixels (full-size sampling).      */
int hqo_fwd_rows(const hqo_problem *p, const int8_t *X, int zx, const int8_t *Wt,
                 const int64_t *rows, int64_t nrows, int32_t *c)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < nrows; i++) bad |= fwd_row(p, X, zx, Wt, rows[i], c + i * p->Cout);
    return bad;
}

/* Input gradient, Sec. 3.1, written as the literal adjoint of the forward
 * sum: every (output pixel, tap) pair adds into the input pixel it read.     */
int hqo_dgrad(const hqo_problem *p, const int8_t *dY, int zg, const int8_t *Wt, int32_t *c)
{
    int OH, OW; hqo_out_hw(p, &OH, &OW);
    int64_t per_img = (int64_t)p->H * p->W * p->C;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int b = 0; b < p->B; b++) {
        int64_t *acc = (int64_t *)calloc((size_t)per_img, sizeof(int64_t));
        for (int oh = 0; oh < OH; oh++)
        for (int ow = 0; ow < OW; ow++) {
            const int8_t *g = dY + (((int64_t)b * OH + oh) * OW + ow) * p->Cout;
            for (int r = 0; r < p->R; r++) {
                int ih = oh * p->stride - p->pad + r;
                if (ih < 0 || ih >= p->H) continue;
                for (int s = 0; s < p->S; s++) {
                    int iw = ow * p->stride - p->pad + s;
                    if (iw < 0 || iw >= p->W) continue;
                    int64_t *a = acc + ((int64_t)ih * p->W + iw) * p->C;
                    if (p->kind == 2) {
                        const int8_t *w = Wt + ((int64_t)r * p->S + s) * p->C;
                        for (int ch = 0; ch < p->C; ch++) a[ch] += (int64_t)((int)g[ch] - zg) * w[ch];
                    } else {
                        for (int n = 0; n < p->Cout; n++) {
                            int64_t gv = (int)g[n] - zg;
                            const int8_t *w = Wt + (((int64_t)n * p->R + r) * p->S + s) * p->C;
                            for (int ch = 0; ch < p->C; ch++) a[ch] += gv * w[ch];
                        }
                    }
                }
            }
        }
        for (int64_t i = 0; i < per_img; i++) {
            if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) bad = 1;
            c[(int64_t)b * per_img + i] = (int32_t)acc[i];
        }
        free(acc);
    }
    return bad;
}

/* Input gradient at chosen input pixels (rows index [B,H,W]); gather form,
 * used only to sample full-size problems.  Pinned against hqo_dgrad.         */
int hqo_dgrad_rows(const hqo_problem *p, const int8_t *dY, int zg, const int8_t *Wt,
                   const int64_t *rows, int64_t nrows, int32_t *c)
{
    int OH, OW; hqo_out_hw(p, &OH, &OW);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < nrows; i++) {
        int64_t m = rows[i];
        int w = (int)(m % p->W), h = (int)((m / p->W) % p->H), b = (int)(m / ((int64_t)p->W * p->H));
        for (int ch = 0; ch < p->C; ch++) {
            int64_t sum = 0;
            for (int oh = 0; oh < OH; oh++) {
                int r = h - (oh * p->stride - p->pad);
                if (r < 0 || r >= p->R) continue;
                for (int ow = 0; ow < OW; ow++) {
                    int s = w - (ow * p->stride - p->pad);
                    if (s < 0 || s >= p->S) continue;
                    const int8_t *g = dY + (((int64_t)b * OH + oh) * OW + ow) * p->Cout;
                    if (p->kind == 2) {
                        sum += (int64_t)((int)g[ch] - zg) * Wt[((int64_t)r * p->S + s) * p->C + ch];
                    } else {
                        for (int n = 0; n < p->Cout; n++)
                            sum += (int64_t)((int)g[n] - zg) *
                                   Wt[(((int64_t)n * p->R + r) * p->S + s) * p->C + ch];
                    }
                }
            }
            if (sum > INT32_MAX || sum < INT32_MIN) bad = 1;
            c[i * p->C + ch] = (int32_t)sum;
        }
    }
    return bad;
}

/* Weight gradient, Sec. 3.1: c[n,r,s,ch] = sum over the batch and all output
 * pixels of (X~ - z_x)(G~_Y - z_g); depthwise: c[r,s,ch].                     */
int hqo_wgrad(const hqo_problem *p, const int8_t *X, int zx, const int8_t *dY, int zg, int32_t *c)
{
    int OH, OW; hqo_out_hw(p, &OH, &OW);
    int64_t nout = (p->kind == 2 ? 1 : (int64_t)p->Cout) * p->R * p->S * p->C;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t o = 0; o < nout; o++) {
        int ch = (int)(o % p->C);
        int s = (int)((o / p->C) % p->S);
        int r = (int)((o / ((int64_t)p->C * p->S)) % p->R);
        int n = p->kind == 2 ? ch : (int)(o / ((int64_t)p->C * p->S * p->R));
        int64_t sum = 0;
        for (int b = 0; b < p->B; b++)
        for (int oh = 0; oh < OH; oh++) {
            int ih = oh * p->stride - p->pad + r;
            if (ih < 0 || ih >= p->H) continue;
            for (int ow = 0; ow < OW; ow++) {
                int iw = ow * p->stride - p->pad + s;
                if (iw < 0 || iw >= p->W) continue;
                int xv = (int)X[(((int64_t)b * p->H + ih) * p->W + iw) * p->C + ch] - zx;
                int gv = (int)dY[(((int64_t)b * OH + oh) * OW + ow) * p->Cout + n] - zg;
                sum += (int64_t)xv * gv;
            }
        }
        if (sum > INT32_MAX || sum < INT32_MIN) bad = 1;
        c[o] = (int32_t)sum;
    }
    return bad;
}

/* ------------------------------------------------------------------------- */
/* Statistics and quantizers.                                                 */
/* ------------------------------------------------------------------------- */

/* eq. (1) on the accumulator output: exact min and max.                      */
void hqo_minmax(const int32_t *c, int64_t n, int32_t *mn, int32_t *mx)
{
    int32_t lo = INT32_MAX, hi = INT32_MIN;
    for (int64_t i = 0; i < n; i++) { if (c[i] < lo) lo = c[i]; if (c[i] > hi) hi = c[i]; }
    *mn = lo; *mx = hi;
}

/* Quantizer parameters of a range (q_min, q_max).                            */
void hqo_qparams(float qmin, float qmax, int symmetric, int qlo, int qhi, float *scale, int32_t *zp)
{
    if (symmetric) {
        float amax = fmaxf(fabsf(qmin), fabsf(qmax));
        *scale = amax > 0.0f ? amax / (float)qhi : 1.0f;
        *zp = 0;
        return;
    }
    float lo = fminf(qmin, 0.0f), hi = fmaxf(qmax, 0.0f);
    float width = hi - lo;
    float s = width > 0.0f ? width / (float)(qhi - qlo) : 1.0f;
    float q = lo / s;
    float z = rintf((float)qlo - q);
    if (z < (float)qlo) z = (float)qlo;
    if (z > (float)qhi) z = (float)qhi;
    *scale = s; *zp = (int32_t)z;
}

/* Static quantization of accumulator outputs (Sec. 3.2) with a given output
 * quantizer: one fp32 multiply by m = acc_scale / s_y, round half to even,
 * clamp to the grid.  Counts the codes that clamped (saturation, Sec. 4).     */
void hqo_requant(const int32_t *c, int64_t n, float acc_scale, float s_y, int z_y, int qlo, int qhi,
                 int8_t *out, uint64_t *clip_lo, uint64_t *clip_hi)
{
    float m = acc_scale / s_y;
    float flo = (float)(qlo - z_y), fhi = (float)(qhi - z_y);
    uint64_t nlo = 0, nhi = 0;
    for (int64_t i = 0; i < n; i++) {
        float v = (float)c[i];
        float r = rintf(v * m);
        if (r < flo) { r = flo; nlo++; }
        if (r > fhi) { r = fhi; nhi++; }
        out[i] = (int8_t)((int)r + z_y);
    }
    *clip_lo = nlo; *clip_hi = nhi;
}

/* Random bits for stochastic rounding: a counter-based generator, so that any implementation
 * reproduces the same decision for the same (element index, seed).  The low index word goes
 * through the finalizer of MurmurHash3 (two multiply / xor-shift rounds); between its rounds the
 * first key word is added and the high index word (times an odd constant) plus the second key word
 * are folded in; a third multiply (golden-ratio constant) / xor-shift closes.  The key enters after
 * a non-linear step, so two seeds do not give the same stream with relabelled elements.       */
uint32_t hqo_sr_bits(uint64_t idx, uint64_t seed)
{
    uint32_t h = (uint32_t)idx;
    h ^= h >> 16; h *= 0x85ebca6bu; h += (uint32_t)seed;
    h ^= (uint32_t)(idx >> 32) * 0x85ebca77u + (uint32_t)(seed >> 32);
    h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    h *= 0x9e3779b1u; h ^= h >> 15;
    return h;
}

/* Static quantization with stochastic rounding (the paper quantizes gradients this way, Sec. 5
 * experimental setup, after Gupta et al. 2015): x = fp32(c) * m as in hqo_requant, then x is
 * rounded up with probability x - floor(x) and down otherwise: up iff the fraction exceeds
 * u = (top 24 random bits) / 2^24, the draw of element i being hqo_sr_bits(idx0 + i, seed).
 * Clamping and clip counting as in hqo_requant, on the rounded value.                        */
void hqo_requant_sr(const int32_t *c, int64_t n, float acc_scale, float s_y, int z_y, int qlo, int qhi,
                    uint64_t idx0, uint64_t seed, int8_t *out, uint64_t *clip_lo, uint64_t *clip_hi)
{
    float m = acc_scale / s_y;
    float flo = (float)(qlo - z_y), fhi = (float)(qhi - z_y);
    uint64_t nlo = 0, nhi = 0;
    for (int64_t i = 0; i < n; i++) {
        float x = (float)c[i] * m;
        float f = floorf(x);
        float frac = x - f;                                  /* exact */
        float u = (float)(hqo_sr_bits(idx0 + (uint64_t)i, seed) >> 8) * (1.0f / 16777216.0f);
        float r = frac > u ? f + 1.0f : f;
        if (r < flo) { r = flo; nlo++; }
        if (r > fhi) { r = fhi; nhi++; }
        out[i] = (int8_t)((int)r + z_y);
    }
    *clip_lo = nlo; *clip_hi = nhi;
}

/* In-hindsight min-max, eq. (2)-(3), from the minimum and maximum of the tensor in real units;
 * first call sets q^0 (Sec. 4.1).                                             */
void hqo_range_update_real(hqo_range *r, float gmin, float gmax)
{
    if (!r->initialized) {
        r->qmin = gmin; r->qmax = gmax; r->initialized = 1;
    } else {
        float one_minus = 1.0f - r->eta;
        float a = one_minus * gmin, b = r->eta * r->qmin;
        r->qmin = a + b;
        a = one_minus * gmax; b = r->eta * r->qmax;
        r->qmax = a + b;
    }
    hqo_qparams(r->qmin, r->qmax, r->symmetric, r->qlo, r->qhi, &r->scale, &r->zero_point);
}

/* The same from accumulator statistics: one accumulator unit is worth acc_scale.  */
void hqo_range_update(hqo_range *r, int32_t acc_min, int32_t acc_max, float acc_scale)
{
    hqo_range_update_real(r, acc_scale * (float)acc_min, acc_scale * (float)acc_max);
}

/* ------------------------------------------------------------------------- */
/* Saturation-driven range update (Sec. 4: the saturation ratio as the statistic).            */
/* ------------------------------------------------------------------------- */

/* Natural logarithm of a positive normal fp32 number, evaluated with a fixed sequence of fp32
 * operations (each rounded once) so that every implementation of this sequence returns the same
 * bits: x = m * 2^e with m in [sqrt(1/2), sqrt(2)), s = (m - 1) / (m + 1),
 * ln x = e * ln 2 + 2 s (1 + s^2/3 + s^4/5 + s^6/7).  Absolute error below 1e-6.               */
float hqo_ln_fixed(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int e = (int)((bits >> 23) & 0xff) - 127;
    uint32_t mb = (bits & 0x007fffffu) | 0x3f800000u;          /* m in [1, 2) */
    float m;
    memcpy(&m, &mb, 4);
    if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
    float t = m - 1.0f;
    float d = m + 1.0f;
    float sq = t / d;
    float s2 = sq * sq;
    float p = s2 * (1.0f / 7.0f);
    p = p + 0.2f;
    p = p * s2;
    p = p + (1.0f / 3.0f);
    p = p * s2;
    p = p + 1.0f;
    float lm = 2.0f * sq;
    lm = lm * p;
    float le = (float)e * 0.693147182f;
    return le + lm;
}

/* State of the saturation-driven estimator for one quantizer: the acceptable band of the
 * saturation ratio, the ratio to aim at when the range is moved, the number of consecutive
 * iterations the ratio must lie outside the band before that happens, and the running count
 * of such iterations.                                                                         */
typedef struct { float alpha_min, alpha_max, alpha_target; int32_t tau, streak; } hqo_saturation;

/* One iteration of the saturation-driven update (the variant Sec. 4 names next to min-max; the
 * rule below is this build's reading, the paper gives no equation for it):
 *   alpha = (clip_lo + clip_hi) / count                         the saturation ratio of the tensor just quantized
 *   alpha inside [alpha_min, alpha_max]: the range stays, the streak ends
 *   otherwise the streak grows; once it exceeds tau, the range is rescaled about zero by
 *     rho = ln(alpha_target) / ln(alpha^),  alpha^ = clamp(alpha, 1 / (2 count), 1/2),
 *   which for a zero-mean Laplace tensor (tail mass exp(-q / b) beyond q) is the quantile q' =
 *   b ln(1 / alpha_target) with b estimated from the observed ratio: the inverse CDF of the
 *   Laplace distribution, no pass over the data.  The first call (range not initialised) sets
 *   q^0 from the minimum and maximum of the first batch, as Sec. 4.1 does.                     */
void hqo_range_update_saturation(hqo_range *r, hqo_saturation *sat, uint64_t clip_lo, uint64_t clip_hi,
                                 uint64_t count, int32_t acc_min, int32_t acc_max, float acc_scale)
{
    if (count == 0) return;
    if (!r->initialized) {
        r->qmin = acc_scale * (float)acc_min; r->qmax = acc_scale * (float)acc_max; r->initialized = 1;
        sat->streak = 0;
    } else {
        float alpha = (float)(clip_lo + clip_hi) / (float)count;
        if (alpha >= sat->alpha_min && alpha <= sat->alpha_max) {
            sat->streak = 0;
        } else {
            sat->streak += 1;
            if (sat->streak > sat->tau) {
                float floor_ = 0.5f / (float)count;
                float ah = alpha < floor_ ? floor_ : alpha;
                if (ah > 0.5f) ah = 0.5f;
                float rho = hqo_ln_fixed(sat->alpha_target) / hqo_ln_fixed(ah);
                r->qmin = rho * r->qmin;
                r->qmax = rho * r->qmax;
                sat->streak = 0;
            }
        }
    }
    hqo_qparams(r->qmin, r->qmax, r->symmetric, r->qlo, r->qhi, &r->scale, &r->zero_point);
}

/* Static quantization (Sec. 3.2) of a real-valued tensor with a given quantizer (s, z): the
 * arithmetic of hqo_requant with the real value in the accumulator's place and unit 1, so
 * m = 1 / s.  Also returns the tensor's minimum and maximum, which eq. (2)-(3) consume.  */
void hqo_quantize_tensor(const float *x, int64_t n, float s, int z, int qlo, int qhi,
                         int8_t *out, uint64_t *clip_lo, uint64_t *clip_hi, float *xmin, float *xmax)
{
    float m = 1.0f / s;
    float flo = (float)(qlo - z), fhi = (float)(qhi - z);
    uint64_t nlo = 0, nhi = 0;
    for (int64_t i = 0; i < n; i++) {
        float r = rintf(x[i] * m);
        if (r < flo) { r = flo; nlo++; }
        if (r > fhi) { r = fhi; nhi++; }
        out[i] = (int8_t)((int)r + z);
        if (i == 0 || x[i] < *xmin) *xmin = x[i];
        if (i == 0 || x[i] > *xmax) *xmax = x[i];
    }
    *clip_lo = nlo; *clip_hi = nhi;
}

/* The same with stochastic rounding: the decision rule and the draw of hqo_requant_sr
 * (element i of the tensor draws hqo_sr_bits(i, seed)), on y = x * m.                    */
void hqo_quantize_tensor_sr(const float *x, int64_t n, float s, int z, int qlo, int qhi, uint64_t seed,
                            int8_t *out, uint64_t *clip_lo, uint64_t *clip_hi, float *xmin, float *xmax)
{
    float m = 1.0f / s;
    float flo = (float)(qlo - z), fhi = (float)(qhi - z);
    uint64_t nlo = 0, nhi = 0;
    for (int64_t i = 0; i < n; i++) {
        float y = x[i] * m;
        float f = floorf(y);
        float frac = y - f;
        float u = (float)(hqo_sr_bits((uint64_t)i, seed) >> 8) * (1.0f / 16777216.0f);
        float r = frac > u ? f + 1.0f : f;
        if (r < flo) { r = flo; nlo++; }
        if (r > fhi) { r = fhi; nhi++; }
        out[i] = (int8_t)((int)r + z);
        if (i == 0 || x[i] < *xmin) *xmin = x[i];
        if (i == 0 || x[i] > *xmax) *xmax = x[i];
    }
    *clip_lo = nlo; *clip_hi = nhi;
}

/* Q_W (Sec. 3.1): the weight quantizer's range does not depend on the batch; the paper always
 * uses the current min-max of the weight tensor (Sec. 5, experimental setup).  Symmetric 8-bit
 * grid -127..127: s = max|w| / 127 (1 for an all-zero tensor), code = clamp(rne(w / s)), every
 * fp32 operation rounded once.                                                              */
void hqo_quantize_weights(const float *w, int64_t n, int8_t *out, float *scale)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; i++) { float a = fabsf(w[i]); if (a > amax) amax = a; }
    float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    for (int64_t i = 0; i < n; i++) {
        float r = rintf(w[i] / s);
        if (r < -127.0f) r = -127.0f;
        if (r > 127.0f) r = 127.0f;
        out[i] = (int8_t)(int)r;
    }
    *scale = s;
}

/* Weight gradient kept in FP32 (Sec. 3.1): one multiply by s_x * s_g.         */
void hqo_wgrad_scale(const int32_t *c, int64_t n, float sx, float sg, float *dW)
{
    float s = sx * sg;
    for (int64_t i = 0; i < n; i++) dW[i] = s * (float)c[i];
}
