/*
 * hq.h -- C ABI of the in-hindsight quantized-training layer library for MI355X (gfx950).
 *
 * The library runs the three linear operations of a fully quantized layer on 8-bit codes
 * with 32-bit accumulation (paper Sec. 3.1, Fig. 1; Sec. 3.2, Fig. 2) and quantizes each
 * accumulator output in the kernel's epilogue, either
 *   - statically, with the range estimated on earlier iterations, while tracking the
 *     min/max of the current output on the side (in-hindsight min-max, Sec. 4, Sec. 4.1), or
 *   - dynamically, by writing the 32-bit output to memory, deriving the range from it and
 *     reading it back (Sec. 3.2, eq. (1)): the baseline whose traffic eq. (5) counts.
 *
 * General rules
 *   - Every pointer is a DEVICE pointer unless its comment says "host".  The caller owns all
 *     buffers; the library allocates nothing and keeps no state between calls.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and never synchronises with the host.  Quantizer parameters, range state and
 *     statistics live in device memory so that a training step needs no host round trip.
 *   - Return value: HQ_OK or a negative HQ_E_* code.  Shapes the kernels do not support are
 *     reported (HQ_E_BADSHAPE), never padded silently.  Nothing is launched on error.
 *   - Codes are signed 8-bit.  A real value is scale * (code - zero_point).  An unsigned grid
 *     0..255 is stored shifted by -128 together with its zero point.
 *   - Tensors are NHWC, row-major, densely packed, and their base pointers 16-byte aligned.
 *   - Taps of a convolution that fall outside the image hold real zero.
 *   - Weight operands are taken as symmetric (zero point 0); `scale` is the only field of
 *     their hq_qparams that is read.
 *   - Rounding is round-half-to-even in fp32; the multiplier is (s_a * s_b) / s_out with
 *     each operation rounded once.
 */
#ifndef HQ_H
#define HQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HQ_OK            0
#define HQ_E_BADARG    (-1)   /* null / misaligned pointer, bad enum value                  */
#define HQ_E_BADSHAPE  (-2)   /* shape outside what the kernels support (see each call)     */
#define HQ_E_WORKSPACE (-3)   /* workspace missing or smaller than hq_workspace_bytes()     */
#define HQ_E_HIP       (-4)   /* a HIP call failed (launch error)                           */

#define HQ_LINEAR    0        /* out[M,N] = A[M,K] . W[N,K]^T ; problem: B=M, C=K, Cout=N   */
#define HQ_CONV2D    1        /* NHWC convolution as implicit-im2col GEMM                   */
#define HQ_DEPTHWISE 2        /* one R x S filter per channel (Cout == C), no MFMA          */

/* Quantizer parameters that travel with a quantized tensor. */
typedef struct { float scale; int32_t zero_point; } hq_qparams;

/* State of one in-hindsight quantizer (Sec. 4.1).  (qmin, qmax) is the range q^t of
 * eq. (2)-(3) in real units; qp is the quantizer derived from it and is what the fused
 * kernels read.  Asymmetric grid: qlo..qhi = -128..127, range widened to contain 0.
 * Symmetric grid: -127..127, scale = max(|qmin|,|qmax|)/qhi, zero point 0.                 */
typedef struct {
    float      qmin, qmax;
    float      eta;           /* momentum; the paper uses 0.9 (Sec. 5.2)                     */
    int32_t    qlo, qhi;
    int32_t    symmetric;     /* 0 asymmetric, 1 symmetric                                   */
    int32_t    initialized;   /* 0 until q^0 has been set from the first batch (Sec. 4.1)    */
    hq_qparams qp;
} hq_range;

/* Online statistics of one output tensor, gathered from the accumulator before the
 * quantization step (Sec. 4).  acc_min/acc_max are over the zero-point-corrected 32-bit
 * accumulator outputs; one accumulator unit is worth acc_scale in real units.
 * clip_lo/clip_hi count the outputs whose rounded code fell below qlo / above qhi
 * (saturation ratio = (clip_lo + clip_hi) / count, Sec. 4 footnote).
 *
 * A record is sharded: the workgroups of a GEMM merge their minima, maxima and clip counts
 * into one of HQ_STATS_PARTS partial records, each in a 128-byte line of its own, so that
 * the atomics of a launch spread over many addresses instead of queueing on one.  The
 * leading fields are the fold of the partial records: hq_stats_fold, hq_range_update and
 * hq_gemm_dynamic (between its passes) move what the partial records hold into them and
 * empty the partial records, so folding twice is harmless.  acc_scale and count are
 * written by the GEMMs directly.  hq_stats_reset / hq_range_update empty the whole record. */
#define HQ_STATS_PARTS 64
typedef struct {
    int32_t  acc_min, acc_max;
    uint64_t clip_lo, clip_hi;
    uint8_t  pad[104];
} hq_stats_part;                                   /* 128 bytes */
typedef struct {
    int32_t  acc_min, acc_max;
    float    acc_scale;
    uint32_t fp32_keys;       /* 0: accumulator units (the GEMMs); 1: see hq_tensor_quantize */
    uint64_t clip_lo, clip_hi, count;
    uint8_t  pad[88];
    hq_stats_part part[HQ_STATS_PARTS];
} hq_stats;                                        /* 128 + 64 * 128 bytes, 128-byte aligned */

/* Layer shape (host struct).  Linear: kind=HQ_LINEAR, B=M, C=K, Cout=N, H=W=R=S=stride=1,
 * pad=0.  Output spatial size: OH = (H + 2*pad - R)/stride + 1, same for OW.
 * Layouts:  X  [B][H][W][C]           dY [B][OH][OW][Cout]
 *           W  [Cout][R][S][C]        (depthwise: [R][S][C])
 *           Wd [C][R][S][Cout]        the same weights re-laid for hq_gemm_dgrad (depthwise: = W)
 * Supported: C % 4 == 0 and Cout % 4 == 0 for HQ_LINEAR / HQ_CONV2D (full-rate path when the
 * reduced channel count is a multiple of 16); C % 4 == 0 for HQ_DEPTHWISE; B*H*W and
 * B*OH*OW below 2^31.  In addition HQ_CONV2D takes C == 3 (a network's first layer on RGB images,
 * pixels of 3 bytes) with a filter row of S * 3 <= 32 bytes:
 *   hq_gemm_fwd, hq_gemm_dynamic (forward)   filters of at most 7 rows, Cout a multiple of 16 up to 64;
 *   hq_gemm_wgrad, hq_gemm_wgrad_update,
 *   hq_gemm_wgrad_static, hq_weight_prepare  any R, any Cout that is a multiple of 4;
 *   hq_gemm_dgrad, the stochastic-rounding entries   refused: a first layer has no input gradient.
 * Anything outside these limits returns HQ_E_BADSHAPE.                                          */
typedef struct {
    int32_t kind;
    int32_t B, H, W, C;
    int32_t R, S, stride, pad;
    int32_t Cout;
} hq_problem;

/* Entry indices for hq_workspace_bytes. */
#define HQ_ENTRY_FWD      0
#define HQ_ENTRY_DGRAD    1
#define HQ_ENTRY_WGRAD    2
#define HQ_ENTRY_DYNAMIC_FWD   3
#define HQ_ENTRY_DYNAMIC_DGRAD 4

/* Bytes of device workspace an entry point needs for this problem (host, pure; 0 = none).
 * Returns 0 also for an invalid problem; the entry point itself reports the error.          */
size_t hq_workspace_bytes(int32_t entry, const hq_problem *p /* host */);

/* Forward Y~ = Q_Y(X~ . W~) with in-hindsight static quantization (Sec. 3.1 forward pass;
 * Sec. 3.2 static quantization; Sec. 4 steps 1 and 2).
 *   X, xq    input codes and their quantizer (xq->zero_point may be non-zero)
 *   W, wq    weight codes [Cout][R][S][C] (depthwise [R][S][C]) and their scale
 *   wsum     int32 [Cout]: sum of the weight codes of each output channel, from
 *            hq_weight_prepare; used to remove the input zero point
 *   yr       range state q^t of the output quantizer, read only (must be initialized)
 *   Y        output codes [B][OH][OW][Cout], written once
 *   yq       out: the quantizer actually used for Y (a copy of yr->qp), so that consumers
 *            never race with a later hq_range_update
 *   st       statistics of this output, merged in place (min, max, clips into the partial
 *            records, count) and st->acc_scale set to xq->scale * wq->scale                  */
int hq_gemm_fwd(const hq_problem *p /* host */,
                const int8_t *X, const hq_qparams *xq,
                const int8_t *W, const hq_qparams *wq, const int32_t *wsum,
                const hq_range *yr, int8_t *Y, hq_qparams *yq, hq_stats *st, void *stream);

/* Input gradient G~_X = Q_G(G~_Y . W~^T), same epilogue as the forward pass with the
 * gradient quantizer's own range state (Sec. 3.1 backward pass).
 *   dY, gq   output-gradient codes [B][OH][OW][Cout] and their quantizer
 *   Wd, wq   weights in [C][R][S][Cout] order (depthwise: [R][S][C]) and their scale
 *   wdsum    int32 [C]: sum over (r,s,cout) of the weight codes of each input channel
 *   gr       range state of Q_G, read only;  dX [B][H][W][C];  dxq, st as in hq_gemm_fwd    */
int hq_gemm_dgrad(const hq_problem *p /* host */,
                  const int8_t *dY, const hq_qparams *gq,
                  const int8_t *Wd, const hq_qparams *wq, const int32_t *wdsum,
                  const hq_range *gr, int8_t *dX, hq_qparams *dxq, hq_stats *st, void *stream);

/* hq_gemm_dgrad with STOCHASTIC ROUNDING in the epilogue: the paper quantizes the activation
 * gradient this way in all its experiments (Sec. 5, experimental setup, and the gradient-
 * quantization paragraph; after Gupta et al. 2015).  The scaled accumulator x = fp32(c) * m is
 * rounded up with probability x - floor(x): up iff that fraction exceeds u = r / 2^24, r being the
 * top 24 of 32 random bits drawn for the element from a counter-based generator keyed on
 * (linear index of the element in dX, seed).  The result therefore depends on the seed and the
 * tensor only, not on the kernel's tiling; callers derive `seed` (host value) from their base
 * seed, the tensor and the iteration.  Clamping, clip counts, statistics and all other arguments
 * as hq_gemm_dgrad.  Same kernel selection as hq_gemm_dgrad, except that HQ_DEPTHWISE layers
 * always take the general stencil.                                                           */
int hq_gemm_dgrad_sr(const hq_problem *p /* host */,
                     const int8_t *dY, const hq_qparams *gq,
                     const int8_t *Wd, const hq_qparams *wq, const int32_t *wdsum,
                     const hq_range *gr, uint64_t seed,
                     int8_t *dX, hq_qparams *dxq, hq_stats *st, void *stream);

/* Weight gradient G_W = X~^T . G~_Y, kept in FP32 (Sec. 3.1): no quantizer, no range state.
 *   X, xq / dY, gq   both operands may carry a non-zero zero point
 *   dW       fp32, shaped like W: (xq->scale * gq->scale) * float(integer sum)
 *   dW_acc   optional int32 copy of the zero-point-free integer sum (NULL to skip)
 *   ws       workspace of hq_workspace_bytes(HQ_ENTRY_WGRAD, p) bytes, 16-byte aligned;
 *            contents are scratch                                                            */
int hq_gemm_wgrad(const hq_problem *p /* host */,
                  const int8_t *X, const hq_qparams *xq,
                  const int8_t *dY, const hq_qparams *gq,
                  float *dW, int32_t *dW_acc, void *ws, size_t ws_bytes, void *stream);

/* hq_gemm_wgrad for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the workspace is a fixed array of
 * HQ_STATIC_SCRATCH_BYTES that the library itself holds on every GPU it is loaded on, from load
 * until the process ends.  No allocation happens in this call or below it.  Same kernels, same
 * results and same remaining arguments as hq_gemm_wgrad.
 *   - Problems with hq_workspace_bytes(HQ_ENTRY_WGRAD, p) > HQ_STATIC_SCRATCH_BYTES are refused
 *     with HQ_E_WORKSPACE and nothing is launched.
 *   - All calls on one GPU share that GPU's array (each call clears what it needs at zero, the
 *     rest is overwritten before it is read): calls that overlap in time on one GPU, e.g. on two
 *     streams, race; calls on one stream, or otherwise ordered, do not.                        */
#define HQ_STATIC_SCRATCH_BYTES (64u << 20)
int hq_gemm_wgrad_static(const hq_problem *p /* host */,
                         const int8_t *X, const hq_qparams *xq,
                         const int8_t *dY, const hq_qparams *gq,
                         float *dW, int32_t *dW_acc, void *stream);

/* hq_gemm_wgrad followed by hq_range_update_batch(r, st, n) in one call: the range updates run as
 * n extra workgroups of the call's last launch, next to its own work, instead of in a launch of
 * their own.  For the layer step fwd, dgrad, wgrad: the statistics must come from launches earlier
 * on the stream (the forward and input-gradient GEMMs); the weight gradient itself reads no range.
 * 1 <= n <= 4096; all other arguments and the result as hq_gemm_wgrad.                          */
int hq_gemm_wgrad_update(const hq_problem *p /* host */,
                         const int8_t *X, const hq_qparams *xq,
                         const int8_t *dY, const hq_qparams *gq,
                         float *dW, int32_t *dW_acc, void *ws, size_t ws_bytes,
                         hq_range *r, hq_stats *st, int32_t n, void *stream);

/* In-hindsight min-max update, eq. (2)-(3): folds the statistics of the tensor just
 * produced into the range for the next iteration and re-derives r->qp.  If r is not
 * initialized the statistics become q^0 (Sec. 4.1).  Folds the partial records first and
 * empties *st afterwards.  With st->count == 0 the range is left as it is.  One wavefront;
 * run it on the stream that produced the tensor, any time after the producing kernel.        */
int hq_range_update(hq_range *r, hq_stats *st, void *stream);

/* State of the saturation-driven estimator of one quantizer (Sec. 4 names the saturation ratio, the
 * share of values outside the quantization grid, as the other statistic that is cheap to take at
 * the accumulator): the band the ratio may lie in, the ratio to aim at when the range is moved, how
 * many iterations in a row the ratio must lie outside the band before that happens (tau), and the
 * running count of such iterations (streak, start at 0).                                      */
typedef struct {
    float   alpha_min, alpha_max, alpha_target;
    int32_t tau, streak;
} hq_saturation;

/* Saturation-driven range update for n quantizers (arrays r[n], st[n], sat[n]), one launch, to be
 * called where hq_range_update would be.  The paper gives no equation for this variant; the rule:
 *   alpha = (clip_lo + clip_hi) / count of the tensor just quantized (fp32)
 *   alpha_min <= alpha <= alpha_max: the range stays, streak = 0
 *   otherwise streak += 1, and once streak > tau the range is rescaled about zero,
 *     (qmin, qmax) *= ln(alpha_target) / ln(clamp(alpha, 1 / (2 count), 1/2)),   streak = 0:
 *   for a zero-mean Laplace tensor with scale b a share exp(-q / b) lies beyond +-q, so this is the
 *   quantile b ln(1 / alpha_target) with b taken from the observed ratio (the inverse CDF of the
 *   Laplace distribution; no pass over the data).  ln is evaluated by a fixed sequence of fp32
 *   operations (exponent plus an odd polynomial in (m - 1) / (m + 1)), each rounded once.
 * A range that is not initialized takes q^0 from the minimum and maximum in st, as
 * hq_range_update does (Sec. 4.1).  r->qp is re-derived, st is folded first and emptied afterwards;
 * with st->count == 0 nothing changes.  The statistics must come from GEMM outputs
 * (fp32_keys == 0).                                                                           */
int hq_range_update_saturation(hq_range *r, hq_stats *st, hq_saturation *sat, int32_t n, void *stream);

/* The same update for n quantizers in one launch: r[i] is updated from st[i], i < n (arrays of
 * records).  A tensor's range is read next by its own layer's launch of the following iteration,
 * so a training step can keep the range states of all its tensors in one array and update them
 * together after the sweep instead of paying one small launch per tensor.                     */
int hq_range_update_batch(hq_range *r, hq_stats *st, int32_t n, void *stream);

/* Dynamic-quantization baseline (Sec. 3.2; eq. (1); traffic of eq. (5)): pass 1 runs the
 * same GEMM and writes every zero-point-corrected 32-bit output to `ws` while gathering
 * min/max; a one-wavefront kernel folds the statistics and derives the quantizer; pass 2 reads the 32-bit tensor back,
 * quantizes and writes the codes.
 *   op        HQ_ENTRY_DYNAMIC_FWD (A=X, Bw=W, bsum=wsum) or HQ_ENTRY_DYNAMIC_DGRAD
 *             (A=dY, Bw=Wd, bsum=wdsum)
 *   mode      HQ_DYN_CURRENT: range = min-max of this tensor, eq. (1); r's (qmin,qmax) are
 *             touched only if r is not initialized, in which case they become q^0 (Sec. 4.1).
 *             HQ_DYN_RUNNING: running min-max (Sec. 4.1, last paragraph): r is first moved by
 *             eq. (2)-(3) with THIS tensor's statistics, then used to quantize it.
 *   r         supplies the grid (qlo, qhi, symmetric) and eta; see `mode` for what is written
 *   st        as in hq_gemm_fwd.  HQ_DYN_CURRENT leaves it filled, so that hq_range_update can follow
 *             and move r by eq. (2)-(3).  HQ_DYN_RUNNING has already moved r with these statistics:
 *             follow it with hq_stats_reset, not hq_range_update (which would apply the same
 *             minimum and maximum to r a second time)
 *   ws        >= hq_workspace_bytes(op, p) bytes: the 32-bit round trip                     */
#define HQ_DYN_CURRENT 0
#define HQ_DYN_RUNNING 1
int hq_gemm_dynamic(int32_t op, int32_t mode, const hq_problem *p /* host */,
                    const int8_t *A, const hq_qparams *aq,
                    const int8_t *Bw, const hq_qparams *bq, const int32_t *bsum,
                    hq_range *r, int8_t *out, hq_qparams *outq, hq_stats *st,
                    void *ws, size_t ws_bytes, void *stream);

/* hq_gemm_dynamic with stochastic rounding in the second pass (the dynamic estimators with the
 * paper's gradient rounding, Sec. 5.1 / 5.2): decision rule, generator and element index as in
 * hq_gemm_dgrad_sr.  All other arguments as hq_gemm_dynamic.                                   */
int hq_gemm_dynamic_sr(int32_t op, int32_t mode, const hq_problem *p /* host */,
                       const int8_t *A, const hq_qparams *aq,
                       const int8_t *Bw, const hq_qparams *bq, const int32_t *bsum,
                       hq_range *r, uint64_t seed, int8_t *out, hq_qparams *outq, hq_stats *st,
                       void *ws, size_t ws_bytes, void *stream);

/* Empties n statistics records (min = INT32_MAX, max = INT32_MIN, counters 0). */
int hq_stats_reset(hq_stats *st, int32_t n, void *stream);

/* Folds the partial records of n statistics records into their leading fields (and empties
 * the partial records), so that a reader of acc_min / acc_max / clip_lo / clip_hi sees
 * everything the kernels before it on the stream have merged.                               */
int hq_stats_fold(hq_stats *st, int32_t n, void *stream);

/* Weight-side preparation, once per weight update (the weight quantizer's output does not
 * depend on the batch, Sec. 3.1): from W [Cout][R][S][C] writes the dgrad layout
 * Wd [C][R][S][Cout] (skipped if Wd is NULL or the layer is depthwise), wsum [Cout] and
 * wdsum [C] (each skipped if NULL).  Depthwise: wsum == wdsum == per-channel tap sum.         */
int hq_weight_prepare(const hq_problem *p /* host */, const int8_t *W,
                      int8_t *Wd, int32_t *wsum, int32_t *wdsum, void *stream);

/* Q_W, the weight quantizer (Sec. 3.1: its range does not depend on the batch; Sec. 5.2: weights
 * take the min-max of the tensor as it is now): symmetric 8-bit quantization of an
 * FP32 tensor with its own range, s = max|w| / 127 (1 for an all-zero tensor),
 * code = clamp(rne(w / s), -127, 127), each fp32 operation rounded once.  Element-wise: Wf and
 * Wq [n] in any layout (follow with hq_weight_prepare for the dgrad layout and the sums).
 * wq receives {s, 0}.  Finite inputs are assumed.                                             */
int hq_weight_quantize(const float *Wf, size_t n, int8_t *Wq, hq_qparams *wq, void *stream);

/* In-hindsight quantization of a real-valued tensor that no GEMM of this library produced (the
 * output of a normalisation or activation layer, a loss gradient), so that a chain of layers runs
 * without the host: static quantization (Sec. 3.2) with the quantizer r->qp that eq. (2)-(3)
 * pre-computed, one pass over X (4 bytes read, 1 byte written per element).  A real value is
 * treated as an accumulator output of unit 1: code = clamp(rne(x * m), qlo - z, qhi - z) + z
 * with m = 1 / s, each fp32 operation rounded once, as in the fused epilogue of the GEMMs.
 *   X [n] fp32 and Q [n] codes, 16-byte aligned, any layout (element-wise); n may be 0
 *   q_out  receives r->qp (travels with Q)
 *   st     minimum and maximum of X, the clip counts and the element count are merged into it; the
 *          minimum and maximum are held as order-preserving integer keys of the fp32 values and
 *          st->fp32_keys is set to 1, which hq_range_update reads; a record serves either real-valued
 *          tensors or GEMM outputs between two updates, not both
 * While r is not initialized its quantizer is {1, 0}: take hq_tensor_quantize_dynamic for the
 * first batch (Sec. 4.1).  Finite inputs are assumed.                                          */
int hq_tensor_quantize(const float *X, size_t n, const hq_range *r, int8_t *Q, hq_qparams *q_out,
                       hq_stats *st, void *stream);

/* hq_tensor_quantize with stochastic rounding (the paper's gradient quantizer, Sec. 5.1 / 5.2):
 * x * m rounds up with probability equal to its fractional part, the draw as in hq_gemm_dgrad_sr
 * with the element's index in X as the counter.  Everything else as hq_tensor_quantize.       */
int hq_tensor_quantize_sr(const float *X, size_t n, const hq_range *r, uint64_t seed, int8_t *Q,
                          hq_qparams *q_out, hq_stats *st, void *stream);

/* The dynamic counterpart (eq. (1)): a first pass reads X for its minimum and maximum, a
 * one-wavefront kernel derives the quantizer, a second pass reads X again and writes the codes
 * (8 bytes read, 1 byte written per element).  mode, r, st as for hq_gemm_dynamic: HQ_DYN_CURRENT
 * quantizes with this tensor's own range and sets q^0 if r is not initialized; HQ_DYN_RUNNING
 * moves r by eq. (2)-(3) with this tensor first and quantizes with the result.  st is left
 * filled: after HQ_DYN_CURRENT hq_range_update can follow, after HQ_DYN_RUNNING hq_stats_reset
 * (the range has already taken these statistics in).  With n == 0, q_out receives r->qp and r is
 * untouched.                                                                                   */
int hq_tensor_quantize_dynamic(int32_t mode, const float *X, size_t n, hq_range *r, int8_t *Q,
                               hq_qparams *q_out, hq_stats *st, void *stream);

/* Measurement aid, not part of the method: launches a kernel in which every wavefront issues
 * iters * 8 int8 MFMAs (32x32x32, operands and accumulators in registers, no memory traffic
 * except one 4-byte store per lane to sink [blocks * 256] at the end).  Timed by the caller, it
 * gives the int8 MFMA rate this device sustains: blocks * 4 * iters * 8 * 2 * 32^3 operations.
 * blocks in 1 .. 65536, iters in 1 .. 2^20.                                                   */
int hq_probe_mfma_rate(int32_t blocks, int32_t iters, int32_t *sink, void *stream);

/* Static text for a return code (host pointer, never NULL). */
const char *hq_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* HQ_H */
