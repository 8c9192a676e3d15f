/*
 * granq.h -- C ABI of the GranQ activation fake-quantizer for AMD MI355X (gfx950).
 *
 * The library implements the activation quantizer of GranQ (arXiv 2503.18339,
 * Alg. 1 without its final accumulation): for a dense NCHW activation tensor
 *
 *   1. granq_range_reduce   per-channel minimum / maximum            (Eq. 4)
 *   2. granq_prescale       per-channel scale and zero-point vectors (Eq. 5)
 *   3. granq_fakequant_fwd  quantize, clamp, dequantize each element (Eq. 1, 6)
 *   4. granq_fakequant_bwd  straight-through-estimator gradient      (Sec. 2.1)
 *
 * Common conventions
 * ------------------
 *  - Every data pointer is a DEVICE pointer owned by the caller; the library
 *    never allocates, frees or keeps a pointer after the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call only enqueues kernels on that stream and returns without
 *    synchronising; results are ready when the stream reaches that point.
 *  - Tensors are dense, contiguous NCHW: element (n,c,h,w) of a tensor with
 *    descriptor {n,c,h,w} lives at index ((n*C + c)*H + h)*W + w.  x, x_hat, dy
 *    and dx of one call share the descriptor's dtype; range, scale and
 *    zero-point vectors are always float32 of length C.
 *  - Arithmetic is IEEE-754 binary32 with round-to-nearest-even, each operation
 *    rounded on its own (true division, no fused multiply-add, subnormals
 *    kept).  With bfloat16 or binary16 storage only loads (exact widening) and
 *    stores (round to nearest even; binary16 overflows to infinity) differ.
 *  - Inputs must be finite.  NaN or infinity in x gives unspecified values
 *    (never a fault or a hang).
 *  - Data pointers should be 16-byte aligned and C*H*W*sizeof(element) a
 *    multiple of 16 for the vectorised kernels; anything else is handled by a
 *    slower element-wise path with the same results.  Pointers must be aligned
 *    to their element size.
 *  - Other granularities are views, no extra entry points:
 *      layer-wise (one range per tensor)       desc {1, 1, 1, N*C*H*W}
 *      per sample and channel (Alg. 1's
 *      C x H x W tensor with no batch axis)    desc {1, N*C, H, W}
 *      channel-wise weights, OIHW              desc {1, O, 1, I*kh*kw}
 *      channels-last activations (N,H,W,C)     desc {N*H*W, C, 1, 1}
 *  - Errors: every function returns a granq_status_t.  Arguments are checked on
 *    the host before anything is launched: on GRANQ_ERR_INVALID_ARG,
 *    GRANQ_ERR_UNSUPPORTED and GRANQ_ERR_WORKSPACE nothing has been enqueued.
 *    GRANQ_ERR_HIP (the runtime refused a launch) may follow kernels of the same
 *    call that were already enqueued.  Calls are re-entrant; the library has no
 *    global mutable state (the one exception, granq_range_reduce_noalloc, says so).
 *    Calls may be captured into a HIP graph.
 */
#ifndef GRANQ_H
#define GRANQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRANQ_OK = 0,
    GRANQ_ERR_INVALID_ARG = 1,   /* null pointer, non-positive dimension, bits outside 1..8 */
    GRANQ_ERR_UNSUPPORTED = 2,   /* unknown dtype, misaligned pointer, tensor too large     */
    GRANQ_ERR_WORKSPACE = 3,     /* workspace missing or smaller than required             */
    GRANQ_ERR_HIP = 4            /* the HIP runtime rejected a launch                      */
} granq_status_t;

typedef enum {
    GRANQ_F32 = 0,               /* IEEE binary32 storage */
    GRANQ_BF16 = 1,              /* bfloat16 storage      */
    GRANQ_F16 = 2                /* IEEE binary16 storage */
} granq_dtype_t;

/* Dense contiguous NCHW tensor. */
typedef struct {
    int64_t n, c, h, w;
    granq_dtype_t dtype;
} granq_desc_t;

/* Static string naming a status code (never NULL). */
const char *granq_status_string(granq_status_t status);

/* Library version as a static string. */
const char *granq_version(void);

/*
 * Bytes of device workspace granq_range_reduce needs for this descriptor
 * (host-only, no GPU call).  The workspace holds per-block partial minima and
 * maxima between the two passes of the reduction.
 */
granq_status_t granq_workspace_bytes(const granq_desc_t *desc, size_t *bytes_out);

/*
 * Host-only introspection (no GPU call): how the vectorised kernels would tile
 * this descriptor.  Fills out[0..23] with
 *   [0] 1 if the shape is eligible for the 128-bit column kernels, else 0
 *   [1] rows  [2] row length  [3] elements per channel within a row
 *   [4] columns per block  [5] column tiles  [6] row groups  [7] rows per group
 *   [8] partial slots per column tile  [9] 1 if no 16-byte vector straddles channels
 *   [10..12] multiplier and the two shifts of the column -> channel division
 *   [13] rows per block of the forward  [14] of the backward  [15] their columns per block
 *   [16] true rows glued into one row of the reduction's matrix (1: none; short rows,
 *        e.g. a channels-last tensor seen as {N*H*W, C, 1, 1}, are glued so that a block's
 *        lanes all have a column; [1], [2] are the glued counts, the channel of a column
 *        follows from the column modulo the true row length)
 *   [17] launches granq_calibrate_fakequant_fwd makes for this descriptor when every pointer is
 *        16-byte aligned: 1 (a block per channel), 2 (first pass; forward that finishes the
 *        reduction) or 3  [18] launches of granq_range_reduce / granq_calibrate: 1 or 2
 *   [19..23] zero, reserved
 * of the matrix view (rows x row length) the kernels walk; [1]..[12] and [16] describe
 * the reduction.  For tests and tuning.
 */
granq_status_t granq_plan_describe(const granq_desc_t *desc, int64_t out[24]);

/*
 * Activation decomposition (Eq. 4; Alg. 1's min/max step; Sec. 5.1: channel-wise
 * quantization is done per channel at the batch level):
 *     ch_min[c] = min over (n,h,w) of x[n,c,h,w],   ch_max[c] likewise.
 * x           [in]  device, N*C*H*W elements of desc->dtype
 * ch_min/max  [out] device, C floats each
 * workspace   [tmp] device, at least granq_workspace_bytes() bytes, 16-byte
 *                   aligned; contents before and after the call are garbage
 */
granq_status_t granq_range_reduce(const void *x, const granq_desc_t *desc,
                                  float *ch_min, float *ch_max,
                                  void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * granq_range_reduce for callers that cannot allocate and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * partials live in a scratch array of GRANQ_STATIC_SCRATCH_BYTES (4 MiB) that the library
 * owns statically on every GPU it is loaded on (held until the process ends); the call makes
 * no hipMalloc / hipFree and calls no allocating routine.  Results are bit-identical to
 * granq_range_reduce.
 *  - A descriptor whose granq_workspace_bytes() exceeds the array returns
 *    GRANQ_ERR_WORKSPACE and launches nothing (every activation shape of ResNet-18/-20/-50
 *    and MobileNetV2 at batch 256 needs less than 1 MiB).
 *  - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *    (two streams, two threads) race and give garbage ranges; serialise them.  Nothing in
 *    the array has to be cleared between calls.
 *  - The first call on a device looks up the array's device address (once per device; the
 *    device current at the call must be the stream's); make it before a graph capture.
 */
#define GRANQ_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
granq_status_t granq_range_reduce_noalloc(const void *x, const granq_desc_t *desc,
                                          float *ch_min, float *ch_max, void *stream);

/*
 * Vectorized pre-scaling parameters (Eq. 2 per channel = Eq. 5; Alg. 1's two
 * steps after the min/max), all channels in one launch:
 *     scale[c]      = (ch_max[c] - ch_min[c]) / (2^bits - 1)
 *     zero_point[c] = round_half_even(-ch_min[c] / scale[c])      (stored as float)
 * A channel whose scale comes out zero, subnormal or NaN (max == min: a dead
 * channel) gets scale 1, so that a dead channel reproduces 0 exactly.  A
 * zero-point of -0 is stored as +0.
 * ch_min/max [in] device, c floats;  scale/zero_point [out] device, c floats.
 * bits in 1..8.
 */
granq_status_t granq_prescale(const float *ch_min, const float *ch_max,
                              int64_t c, int bits,
                              float *scale, float *zero_point, void *stream);

/*
 * granq_range_reduce followed by granq_prescale in one call and one launch
 * fewer (Eq. 4, then Eq. 5: Alg. 1 up to its quantize step): the second pass of
 * the reduction applies Eq. 5 to each channel's range as it produces it.  All
 * four output vectors are written and are bit-identical to those of the two
 * separate calls.  Arguments, workspace and errors as for those two.  Worth it
 * for small tensors, where each dependent launch costs as much as the data.
 */
granq_status_t granq_calibrate(const void *x, const granq_desc_t *desc, int bits,
                               float *ch_min, float *ch_max,
                               float *scale, float *zero_point,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * granq_calibrate followed by granq_fakequant_fwd in one call: Alg. 1 up to the
 * accumulation (Eq. 4, 5, 1, 6).  Every output is bit-identical to that of the
 * separate calls; arguments, workspace and errors as for them (x_hat or codes may
 * be NULL, not both).  A tensor whose channel holds at most 128 KB (n*h*w
 * elements: the regime of the paper's own latency table, batch 16 on CIFAR-size
 * maps) is handled in ONE launch, a block per channel; larger tensors on the 16-byte
 * vector path take TWO: the first pass of the reduction, then the forward, whose leading
 * blocks finish the reduction (second pass, Eq. 5), write the four vectors and hand scale
 * and zero-point to the other blocks through the workspace (a block that finds them pending
 * fetches its rows, then polls; after GRANQ_SPIN_LIMIT polls -- environment; default 20000,
 * and 0 for tensors up to 24 MB whose maps hold at least 64 vectors' elements, where waiting
 * costs more than the work; tests set 0 -- it derives them from the partials itself, so no
 * block depends on another one being scheduled); anything else takes the three launches of
 * the two calls.
 */
granq_status_t granq_calibrate_fakequant_fwd(const void *x, const granq_desc_t *desc, int bits,
                                             float *ch_min, float *ch_max,
                                             float *scale, float *zero_point,
                                             void *x_hat, uint8_t *codes_or_null,
                                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same three steps (Eq. 4, 5, 1, 6: Alg. 1 up to the accumulation) in ONE launch for
 * tensors of up to 64 MB: every block keeps its slice of x in registers from the min / max
 * sweep to the quantization, so x is read once (20 instead of 24 bytes per float32 element
 * and training step) and no kernel boundary separates the steps.  Blocks hand partial ranges
 * and the finished scale / zero-point to each other through `state`.  Outputs are
 * bit-identical to granq_calibrate_fakequant_fwd.
 *
 * state  [in/out] device, granq_resident_state_bytes(desc) bytes, 16-byte aligned.  It must be
 *        ZERO before its first use (granq_resident_state_init enqueues a fill kernel, safe to
 *        capture; hipMemset works too) and then belongs to this descriptor: every completed
 *        call leaves it ready for the next call with the same descriptor.  Two calls that
 *        overlap in time must not share a state.  After a failed or aborted launch zero it again.
 * x_hat  must not be x (a block that stops waiting for the others re-reads x; see below).
 *
 * GRANQ_ERR_UNSUPPORTED, with nothing launched, for a tensor this form does not take: larger
 * than 64 MB, rows that are no whole number of 16-byte vectors, pointers not 16-byte aligned,
 * x_hat == x, or a grid that would not fit the GPU at once -- use granq_calibrate_fakequant_fwd
 * then.  granq_resident_state_bytes (host-only) returns the same code for such a descriptor.
 *
 * No block depends on another one being scheduled: a wavefront waits for its channels'
 * parameters for a bounded number of polls (GRANQ_SPIN_LIMIT in the environment, default
 * 20000, about a microsecond each; tests set 0) and then computes the channels' ranges from x
 * itself, with the same result.
 */
granq_status_t granq_resident_state_bytes(const granq_desc_t *desc, size_t *bytes_out);

granq_status_t granq_resident_state_init(void *state, size_t state_bytes, void *stream);

granq_status_t granq_calibrate_fakequant_fwd_resident(const void *x, const granq_desc_t *desc, int bits,
                                                      float *ch_min, float *ch_max,
                                                      float *scale, float *zero_point,
                                                      void *x_hat, uint8_t *codes_or_null,
                                                      void *state, size_t state_bytes, void *stream);

/*
 * Quantize, clamp, dequantize (Eq. 1, then the dequantization of Eq. 6; Alg. 1's
 * "quantize" and "dequantize & pre-scale" steps):
 *     u     = round_half_even(x / scale[c] + zero_point[c])
 *     q     = min(max(u, 0), 2^bits - 1)
 *     x_hat = scale[c] * (q - zero_point[c])
 * The clamp is not in the paper's Eq. 1; it keeps codes inside b bits when the
 * top of the range lands on a rounding tie or when scale / zero-point come
 * from another tensor.
 * x      [in]  device, desc elements
 * x_hat  [out] device, desc elements (may alias x: in-place), or NULL when only the
 *              codes are wanted (the quantize step alone: the input of the
 *              integer-domain convolution below)
 * codes  [out] device, N*C*H*W bytes holding q, or NULL to skip them; x_hat and
 *              codes both NULL is GRANQ_ERR_INVALID_ARG
 */
granq_status_t granq_fakequant_fwd(const void *x, const granq_desc_t *desc,
                                   const float *scale, const float *zero_point,
                                   int bits, void *x_hat, uint8_t *codes_or_null,
                                   void *stream);

/*
 * Straight-through estimator (Sec. 2.1 names it; the formula is this
 * library's): rounding is treated as the identity and the clamp as a gate,
 *     dx = dy   where 0 <= u <= 2^bits - 1   (u as in granq_fakequant_fwd)
 *     dx = 0    elsewhere,
 * with scale and zero-point treated as constants (no gradient flows into the
 * ranges).
 * x, dy [in] device;  dx [out] device (may alias dy).
 */
granq_status_t granq_fakequant_bwd(const void *x, const void *dy,
                                   const granq_desc_t *desc,
                                   const float *scale, const float *zero_point,
                                   int bits, void *dx, void *stream);

/*
 * Gate-bit variant of the forward / backward pair.  The forward already decides,
 * per element, whether the clamp was inactive; stored as one bit per element it
 * lets the backward read dy and E/8 bytes instead of dy and x (8.125 instead of
 * 12 bytes per float32 element), with identical results:
 *     granq_fakequant_fwd_mask  = granq_fakequant_fwd, plus mask
 *     granq_fakequant_bwd_mask(dy, mask) == granq_fakequant_bwd(x, dy, scale, zero_point)
 * for the x, scale, zero_point and bits the mask was made with.
 * mask layout: bit (i & 7) of byte (i >> 3) is 1 where 0 <= u <= 2^bits - 1 for the
 * element with flat NCHW index i; unused high bits of the last byte are 0.
 * granq_mask_bytes (host-only) returns ceil(N*C*H*W / 8).
 * x_hat may alias x; dx may alias dy.
 */
granq_status_t granq_mask_bytes(const granq_desc_t *desc, size_t *bytes_out);

granq_status_t granq_fakequant_fwd_mask(const void *x, const granq_desc_t *desc,
                                        const float *scale, const float *zero_point,
                                        int bits, void *x_hat, uint8_t *mask, void *stream);

granq_status_t granq_fakequant_bwd_mask(const void *dy, const uint8_t *mask,
                                        const granq_desc_t *desc, void *dx, void *stream);

/*
 * Row-wise fake-quantization of many small matrices in one launch -- the paper's
 * channel-wise quantization "for all weights" (Sec. 5.1): an OIHW weight tensor is
 * a matrix of O rows (output channels) by I*kh*kw columns, each row gets its own
 * range, scale and zero-point (Eq. 2) and is quantized and dequantized (Eq. 1, 6).
 * Weight tensors are small, so one block handles one row start to finish (min/max,
 * scale and zero-point, quantize; the second sweep over the row hits the cache)
 * and all tensors of a network share one launch.  Results are identical to
 * granq_range_reduce + granq_prescale + granq_fakequant_fwd on the view
 * {1, rows, 1, row_len} of each item.
 *
 * items: HOST array of `count` descriptors; every pointer inside is a device pointer.
 *   w [in] rows*row_len elements of `dtype`;  w_hat [out] same (may alias w);
 *   scale, zero_point [out] rows floats each.
 * The descriptors are passed to the kernel by value, up to 32 per launch.
 */
typedef struct {
    const void *w;
    void *w_hat;
    float *scale;
    float *zero_point;
    int64_t rows;
    int64_t row_len;
} granq_rowq_item_t;

granq_status_t granq_rowwise_fakequant_multi(const granq_rowq_item_t *items, int count,
                                             granq_dtype_t dtype, int bits, void *stream);

/*
 * Straight-through backward for the same items: dw = dy where 0 <= u <= 2^bits - 1,
 * else 0, with the scale / zero-point the forward stored.
 *   w, dy [in];  dw [out] (may alias dy);  scale, zero_point [in] rows floats each.
 */
typedef struct {
    const void *w;
    const void *dy;
    void *dw;
    const float *scale;
    const float *zero_point;
    int64_t rows;
    int64_t row_len;
} granq_rowq_bwd_item_t;

granq_status_t granq_rowwise_fakequant_bwd_multi(const granq_rowq_bwd_item_t *items, int count,
                                                 granq_dtype_t dtype, int bits, void *stream);

/*
 * Distortion of the fake-quantized tensor, the two figures of the paper's Table 2:
 *     cosine similarity  X.Q / (|X| |Q|)      relative error  |X - Q| / |X|
 * with Q = x_hat computed on the fly from x, scale, zero_point (x is read once,
 * x_hat is never materialised).  Products and differences are formed and summed
 * in binary64.
 * ch_sums  [out] device, C*4 doubles: per channel  sum x*q, sum x^2, sum q^2, sum (x-q)^2
 * layer    [out] device, 6 doubles: the four sums over all channels (added by a fixed
 *                tree), then cosine similarity and relative error of the
 *                whole tensor (0/0 gives NaN)
 * workspace [tmp] device, granq_distortion_workspace_bytes() bytes, 16-byte aligned
 * Sums are deterministic (fixed reduction tree); they differ from a sequential
 * sum by binary64 rounding only.
 */
granq_status_t granq_distortion_workspace_bytes(const granq_desc_t *desc, size_t *bytes_out);

granq_status_t granq_distortion(const void *x, const granq_desc_t *desc,
                                const float *scale, const float *zero_point, int bits,
                                double *ch_sums, double *layer,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Integer-domain accumulation: the 1x1 convolution that consumes the quantized
 * activations, computed from the integer codes (Eq. 3) with the per-channel scale
 * folded into the weights beforehand, so that the sum itself is pure int8 x int8 ->
 * int32 work on the matrix cores:
 *     y[n,o,k] = out_scale[o] * ( sum_c wq[o,c] * code[n,c,k]  -  corr[o] ),   k over H*W
 *
 * granq_fold_weights prepares wq, corr, out_scale from float weights w[o][c] and the
 * activation quantizer's scale / zero-point:
 *     w'[o,c]      = w[o,c] * scale[c]                      (Eq. 3's w_c * s_c)
 *     out_scale[o] = max_c |w'[o,c]| / 127                  (1 if the row is all zero)
 *     wq[o,c]      = clamp(round_half_even(w'[o,c] / out_scale[o]), -127, 127)
 *     corr[o]      = sum_c wq[o,c] * (int) zero_point[c]    (Eq. 3's - z_c, summed once)
 * so that y approximates sum_c w[o,c] * x_hat[n,c,k] (Eq. 6) up to the rounding of w'.  (The
 * symmetric int8 rounding of a whole row is this library's construction, not the paper's: a
 * channel whose scale is far below the row's largest folds to small or zero weights.)
 *   w [in] o*c floats; scale, zero_point [in] c floats; wq [out] o*c int8; corr [out] o
 *   int64, 8-byte aligned (an exact integer sum: with zero-points of magnitude up to 2^24 and
 *   up to 65535 channels it does not fit 32 bits); out_scale [out] o floats.
 *   zero_point must hold integers of magnitude < 2^24, c < 65536.
 *
 * granq_conv1x1_int8: codes [in] N*C*H*W bytes as written by granq_fakequant_fwd (desc
 * gives n, c, h, w; its dtype is ignored); y [out] N*O*H*W floats, NCHW with O channels.
 * The integer expression sum - corr is exact; it is rounded to binary32 once, then scaled.
 * The matrix-core kernels need codes <= 127 (bits <= 7), C a multiple of 16, O a multiple
 * of 32, C*H*W < 2^25 and 16-byte aligned wq; with H*W a multiple of 4 also 4-byte aligned
 * codes and 16-byte aligned y; with any other H*W >= 4 (7 x 7 maps) codes and y need the
 * alignment of one element only.  Anything else runs a plain integer kernel with identical
 * results.
 */
granq_status_t granq_fold_weights(const float *w, const float *scale, const float *zero_point,
                                  int64_t o, int64_t c, int8_t *wq, int64_t *corr,
                                  float *out_scale, void *stream);

granq_status_t granq_conv1x1_int8(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                  const int8_t *wq, const int64_t *corr, const float *out_scale,
                                  int bits, float *y, void *stream);

/*
 * The same convolution with y stored as y_dtype: the binary32 result above is narrowed to
 * bfloat16 or binary16 with round to nearest even on the store (GRANQ_F32: identical to
 * granq_conv1x1_int8).  The output is what bounds this kernel, so 16-bit storage nearly
 * halves its time.  The matrix-core path then needs y 8-byte aligned (H*W a multiple of 4).
 */
granq_status_t granq_conv1x1_int8_as(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                     const int8_t *wq, const int64_t *corr, const float *out_scale,
                                     int bits, granq_dtype_t y_dtype, void *y, void *stream);

/*
 * The accumulation of Eq. 6 itself: the same 1x1 convolution in floating point over the
 * pre-scaled activations x_hat = s_c (q - z_c) that granq_fakequant_fwd wrote,
 *     y[n,o,k] = sum_c w[o,c] * x_hat[n,c,k],   k over H*W,
 * the float-domain counterpart of granq_conv1x1_int8 (which computes Eq. 3's sum from the
 * integer codes).  Products and sums are binary32, in an order the kernel chooses: for
 * operands of magnitude far from the ends of the binary32 range the result lies within
 * (C + 2) * 2^-24 * sum_c |w[o,c] x_hat[n,c,k]| of the exact sum; it is then rounded to y's type.
 *   x_hat [in]  N*C*H*W elements of desc->dtype, NCHW;  w [in] O*C elements of the same type,
 *   row o holding the C weights of output channel o;  y [out] N*O*H*W elements of the same type.
 *   No pointer may alias another.
 * The matrix-core kernel needs C a multiple of 8, O a multiple of 32, H*W >= 4 and w aligned
 * to four elements; with H*W a multiple of 4 also x_hat and y aligned to four elements (with
 * any other H*W the alignment of one element suffices).  Anything else runs a plain kernel
 * (one thread per output, channels in order).  GRANQ_ERR_UNSUPPORTED: O or N >= 65536,
 * C >= 2^24, or a pointer not aligned to its element.
 */
granq_status_t granq_conv1x1_float(const void *x_hat, const granq_desc_t *desc, int64_t o,
                                   const void *w, void *y, void *stream);

/*
 * Codes at their own width: for bits <= 4 the code q of Eq. 1 fits a nibble, and the integer
 * operands of Eq. 3 can be stored two per byte -- half a byte per element written by the
 * quantize step and read by the convolution.
 * Layout: byte i holds the code of the element with flat NCHW index 2i in its low nibble and
 * that of element 2i + 1 in its high nibble; with an odd element count the last high nibble
 * is 0.  granq_packed4_bytes (host-only) returns ceil(N*C*H*W / 2).
 *
 * granq_fakequant_fwd_packed4 = granq_fakequant_fwd with the codes stored that way
 * (bits in 1..4, else GRANQ_ERR_INVALID_ARG).  x_hat may be NULL (codes only: the quantize
 * step alone, 4.5 bytes moved per float32 element) or alias x.  The vectorised kernels need
 * `packed` 2-byte aligned for float32 and 4-byte aligned for 16-bit tensors.
 *
 * granq_conv1x1_int8_packed4 = granq_conv1x1_int8_as reading such codes; identical results.
 * Its matrix-core path needs H*W a multiple of 4 and 2-byte aligned codes besides the
 * conditions above.
 */
granq_status_t granq_packed4_bytes(const granq_desc_t *desc, size_t *bytes_out);

granq_status_t granq_fakequant_fwd_packed4(const void *x, const granq_desc_t *desc,
                                           const float *scale, const float *zero_point, int bits,
                                           void *x_hat_or_null, uint8_t *packed, void *stream);

granq_status_t granq_conv1x1_int8_packed4(const uint8_t *packed, const granq_desc_t *desc, int64_t o,
                                          const int8_t *wq, const int64_t *corr, const float *out_scale,
                                          int bits, granq_dtype_t y_dtype, void *y, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* GRANQ_H */
