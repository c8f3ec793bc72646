// Host-side launchers shared between the translation units of the hq library.
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/hq.h"

// sr_seed: NULL = round to nearest even; otherwise (host pointer) the seed of stochastic rounding.
int hq_launch_gemm(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                   const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                   int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed = nullptr);

// Fast path for layers whose weights fit in LDS; HQ_E_BADSHAPE means "not covered, use hq_launch_gemm".
// sr_seed as for hq_launch_gemm.
int hq_try_launch_band(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                       const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                       int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream,
                       const uint64_t *sr_seed = nullptr);

// Fast path for forward layers with 4 input channels (a network's first layer); HQ_E_BADSHAPE: not covered.
int hq_try_launch_direct(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                         const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                         int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream);

// Fast path for 3x3 stride-1 layers with 128 or more channels on both sides (input patch staged once per
// 64-channel chunk, weights streamed); HQ_E_BADSHAPE: not covered.  sr_seed as for hq_launch_gemm.
int hq_try_launch_bandw(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Bw,
                        const hq_qparams *bq, const int32_t *bsum, const hq_range *range, int8_t *out8,
                        int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream,
                        const uint64_t *sr_seed = nullptr);

// sr_seed as for hq_launch_gemm (stochastic rounding runs in the general stencil kernel).
int hq_launch_depthwise(const hq_problem *p, int dgrad, const int8_t *A, const hq_qparams *aq, const int8_t *Wt,
                        const hq_qparams *bq, const int32_t *wsum, const hq_range *range, int8_t *out8,
                        int32_t *out32, hq_qparams *outq, hq_stats *st, hipStream_t stream, const uint64_t *sr_seed = nullptr);

size_t hq_wgrad_workspace_bytes(const hq_problem *p);

// ride: range updates to run in the call's last launch (NULL: none); see HqRideAlong.
struct HqRideAlong;
int hq_launch_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                    const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, hipStream_t stream,
                    const HqRideAlong *ride = nullptr);

int hq_launch_depthwise_wgrad(const hq_problem *p, const int8_t *X, const hq_qparams *xq, const int8_t *dY,
                              const hq_qparams *gq, float *dW, int32_t *dW_acc, void *ws, hipStream_t stream,
                              const HqRideAlong *ride = nullptr);
