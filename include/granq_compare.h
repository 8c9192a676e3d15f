/*
 * granq_compare.h -- comparison points for the GranQ benchmark (not part of the
 * four-call quantizer library; built into the same shared object).
 *
 * The paper contrasts its method with (i) a channel-wise baseline that derives
 * the scaling factors channel by channel in a loop (Sec. 5.3.2, Table 5 "Channel-
 * wise (Baseline)") and (ii) quantized inference that applies the per-channel
 * scale inside the accumulation loop (Eq. 3) instead of accumulating pre-scaled
 * activations (Eq. 6 / Alg. 1 output).  These entry points implement both so that
 * the benchmark can time them next to the library.  Conventions (device pointers,
 * stream, status codes, dense NCHW) are those of granq.h.  float32 storage only.
 */
#ifndef GRANQ_COMPARE_H
#define GRANQ_COMPARE_H

#include "granq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Channel-by-channel fake-quantization (Sec. 5.3.2's scalar-loop baseline): a
 * host loop over the C channels; each iteration enqueues, for that channel
 * alone, a min/max reduction over its N slabs, a second pass, the scale and
 * zero-point of that one channel (Eq. 2) and the quantize-dequantize of its
 * elements (Eq. 1, Eq. 6): 4*C launches.  Results are identical to
 * granq_range_reduce + granq_prescale + granq_fakequant_fwd.
 * ch_min, ch_max, scale, zero_point: [out] C floats each.
 * workspace: at least 2 * N floats, 16-byte aligned.
 */
granq_status_t granq_cmp_channel_loop_fwd(const float *x, const granq_desc_t *desc, int bits,
                                          float *ch_min, float *ch_max, float *scale,
                                          float *zero_point, float *x_hat,
                                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Weighted channel sum with the scale applied inside the accumulation loop
 * (Eq. 3), from 8-bit codes, one weight per channel, channels added in order:
 *     y[n,k] = sum_c (w_c * s_c) * (code[n,c,k] - z_c)          k over H*W
 * codes: N*C*H*W bytes; y: [out] N*H*W floats.
 */
granq_status_t granq_cmp_accumulate_inloop(const uint8_t *codes, const granq_desc_t *desc,
                                           const float *scale, const float *zero_point,
                                           const float *weight, float *y, void *stream);

/*
 * The same sum over pre-scaled activations (Eq. 6 / Alg. 1's output):
 *     y[n,k] = sum_c w_c * x_hat[n,c,k]
 */
granq_status_t granq_cmp_accumulate_prescaled(const float *x_hat, const granq_desc_t *desc,
                                              const float *weight, float *y, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* GRANQ_COMPARE_H */
