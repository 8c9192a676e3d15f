/*
 * GranQ activation fake-quantizer -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity authority for the HIP
 * library and shares nothing with it: no header, no helper, no table.  Only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 * It is written to be checked against the paper by eye, not to be fast: scalar
 * nested loops, one channel at a time, one element at a time.
 *
 * Arithmetic: IEEE-754 binary32, round-to-nearest-even, every operation
 * rounded on its own (build with -ffp-contract=off, no fast-math), subnormals
 * kept.  The paper names no precision; binary32 is what the quantizer's users
 * feed it, and integer codes are only comparable bit for bit when both sides
 * round the same operations the same way.
 *
 * Tensor layout: dense NCHW, x[n][c][h][w].  The spatial dimensions only ever
 * appear as the product hw = H*W (the paper's reshape of C x H x W into
 * C x (HW), Sec. 4.2.1 "Activation Decomposition").
 *
 * Readings of points the paper leaves open (each is repeated where it is used):
 *   - the per-channel range runs over batch and space, (n,h,w)   [Sec. 5.1]
 *   - the rounding bracket is round-half-to-even                  [Eq. 1, 2]
 *   - codes are clamped to [0, 2^b - 1] after rounding            [not in Eq. 1]
 *   - a channel whose scale is zero, subnormal or NaN uses scale 1
 *   - zero-point -0 is stored as +0
 *   - the straight-through estimator passes the gradient where the clamp was
 *     inactive and treats scale / zero-point as constants          [Sec. 2.1]
 * Parity unpinned with respect to the authors' own code for the first, fourth
 * and last of these: the paper gives nothing that could confirm them.
 *
 * dtype: 0 = binary32 storage, 1 = bfloat16 storage (uint16 bit patterns),
 * 2 = IEEE binary16 storage (uint16 bit patterns).
 * With 16-bit storage only loads and stores change: a load widens exactly,
 * a store rounds to nearest even; ranges, scale, zero-point and all arithmetic
 * stay binary32.
 */
#include <math.h>
#include <float.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

/* bfloat16 is the top half of a binary32: widening appends 16 zero bits. */
static float bf16_widen(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

/* Narrow a finite binary32 to bfloat16, round to nearest, ties to even:
 * look at the 16 bits that are dropped; above half -> up, below half -> down,
 * exactly half -> towards the even kept pattern.  A carry out of the mantissa
 * moves into the exponent, which is the correct next value. */
static uint16_t bf16_narrow(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    uint32_t kept = bits >> 16;
    uint32_t dropped = bits & 0xFFFFu;
    if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u)))
        kept += 1u;
    return (uint16_t)kept;
}

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits, bias 15) to binary32:
 * every binary16 value is a binary32 value.  value = (-1)^sign * fraction/1024 *
 * 2^-14 for exponent field 0 (zero and subnormals), (1 + fraction/1024) *
 * 2^(exponent-15) for fields 1..30; field 31 is infinity (fraction 0) or NaN. */
static float f16_widen(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exponent = (h >> 10) & 0x1F;
    int fraction = h & 0x3FF;
    float magnitude;
    if (exponent == 0)
        magnitude = ldexpf((float)fraction, -24);
    else if (exponent == 31)
        magnitude = fraction ? NAN : INFINITY;
    else
        magnitude = ldexpf((float)(1024 + fraction), exponent - 25);
    return sign ? -magnitude : magnitude;
}

/* Narrow a binary32 to binary16, round to nearest, ties to even.  The binary16
 * grid around |f| has spacing 2^(e-10) with e = max(floor(log2|f|), -14); the
 * quotient |f| / spacing is computed exactly (a power-of-two scaling of a
 * binary32 that needs at most 24 bits here), rounded to an integer with ties
 * to even, and scaled back.  A result of 2^16 or more is beyond the largest
 * finite binary16 (65504) and becomes infinity. */
static uint16_t f16_narrow(float f)
{
    uint16_t sign = signbit(f) ? 0x8000u : 0u;
    float a = fabsf(f);
    if (isnan(a))
        return (uint16_t)(sign | 0x7E00u);
    if (a == 0.0f)
        return sign;
    if (isinf(a))
        return (uint16_t)(sign | 0x7C00u);
    int e;
    (void)frexpf(a, &e);            /* a = m * 2^e with m in [0.5, 1) */
    e -= 1;                         /* floor(log2 a) */
    if (e < -14)
        e = -14;
    if (e > 16)
        return (uint16_t)(sign | 0x7C00u);
    double steps = rint(ldexp((double)a, 10 - e));   /* exact scaling; rint under FE_TONEAREST ties to even */
    /* steps is in [0, 2048]; 2048 means the next binade */
    if (e == -14 && steps < 1024.0)
        return (uint16_t)(sign | (uint16_t)steps);                 /* subnormal or zero */
    if (steps >= 2048.0) {
        steps = 1024.0;
        e += 1;
    }
    if (e > 15)
        return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)steps - 1024));
}

static float load_elem(const void *base, int64_t i, int dtype)
{
    if (dtype == ORACLE_BF16)
        return bf16_widen(((const uint16_t *)base)[i]);
    if (dtype == ORACLE_F16)
        return f16_widen(((const uint16_t *)base)[i]);
    return ((const float *)base)[i];
}

static void store_elem(void *base, int64_t i, int dtype, float v)
{
    if (dtype == ORACLE_BF16)
        ((uint16_t *)base)[i] = bf16_narrow(v);
    else if (dtype == ORACLE_F16)
        ((uint16_t *)base)[i] = f16_narrow(v);
    else
        ((float *)base)[i] = v;
}

/* Test hooks for the two binary16 conversions (pinned against an independent
 * implementation in the tests). */
void granq_oracle_f16_widen(const uint16_t *h, int64_t count, float *out)
{
    for (int64_t i = 0; i < count; ++i)
        out[i] = f16_widen(h[i]);
}

void granq_oracle_f16_narrow(const float *f, int64_t count, uint16_t *out)
{
    for (int64_t i = 0; i < count; ++i)
        out[i] = f16_narrow(f[i]);
}

/* Largest code, 2^b - 1, as a float (Eq. 2 denominator). */
static float code_max(int bits)
{
    return (float)((1 << bits) - 1);
}

/*
 * Activation decomposition (Eq. 4; Alg. 1, the min/max step): per-channel
 * minimum and maximum.  The paper's tensor has no batch axis; with a batch the
 * statistics are taken "per channel at the batch level" (Sec. 5.1), i.e. over
 * n as well as (h,w), giving one range per channel.
 */
void granq_oracle_range_reduce(const void *x, int dtype,
                               int64_t n, int64_t c, int64_t hw,
                               float *ch_min, float *ch_max)
{
    for (int64_t ic = 0; ic < c; ++ic) {
        float mn = INFINITY;
        float mx = -INFINITY;
        for (int64_t in = 0; in < n; ++in) {
            for (int64_t k = 0; k < hw; ++k) {
                float v = load_elem(x, (in * c + ic) * hw + k, dtype);
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
        }
        ch_min[ic] = mn;
        ch_max[ic] = mx;
    }
}

/*
 * Vectorized scale / zero-point (Eq. 2 per channel = Eq. 5; Alg. 1, the two
 * steps after the min/max):
 *     s_c = (max_c - min_c) / (2^b - 1)
 *     z_c = round(-min_c / s_c)
 * A channel with max == min (a dead post-ReLU channel) would divide by zero;
 * the paper is silent.  Reading: when s is zero, subnormal or NaN it is
 * replaced by 1, so a dead channel reproduces 0 exactly.  "+ 0.0f" turns a
 * zero-point of -0 (min = +0) into +0.
 */
void granq_oracle_prescale(const float *ch_min, const float *ch_max,
                           int64_t c, int bits, float *scale, float *zero_point)
{
    float qmax = code_max(bits);
    for (int64_t ic = 0; ic < c; ++ic) {
        float range = ch_max[ic] - ch_min[ic];
        float s = range / qmax;
        if (!(s >= FLT_MIN))
            s = 1.0f;
        float z = rintf((-ch_min[ic]) / s) + 0.0f;
        scale[ic] = s;
        zero_point[ic] = z;
    }
}

/* The unclamped code of one element: Eq. 1, round(x / s + z). */
static float raw_code(float x, float s, float z)
{
    float t = x / s;
    float v = t + z;
    return rintf(v);
}

/* Codes are kept inside b bits: clamp to [0, 2^b - 1] (a reading taken here; the clamp is not in Eq. 1). */
static float clamp_code(float u, float qmax)
{
    return fminf(fmaxf(u, 0.0f), qmax);
}

/* Dequantization of Eq. 6 (Alg. 1, "dequantize & pre-scale"): s * (q - z). */
static float dequantize(float q, float s, float z)
{
    float d = q - z;
    return s * d;
}

/*
 * Quantize, clamp, dequantize (Eq. 1 then the dequantization of Eq. 6; Alg. 1,
 * the quantize and the "dequantize & pre-scale" steps):
 *     u     = round(x / s_c + z_c)
 *     q     = clamp(u, 0, 2^b - 1)         (the clamp is a reading taken here, not in the paper)
 *     x_hat = s_c * (q - z_c)
 * codes may be NULL.
 */
void granq_oracle_fakequant_fwd(const void *x, int dtype,
                                int64_t n, int64_t c, int64_t hw,
                                const float *scale, const float *zero_point,
                                int bits, void *x_hat, uint8_t *codes)
{
    float qmax = code_max(bits);
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t ic = 0; ic < c; ++ic) {
            float s = scale[ic];
            float z = zero_point[ic];
            for (int64_t k = 0; k < hw; ++k) {
                int64_t i = (in * c + ic) * hw + k;
                float u = raw_code(load_elem(x, i, dtype), s, z);
                float q = clamp_code(u, qmax);
                if (codes)
                    codes[i] = (uint8_t)q;
                store_elem(x_hat, i, dtype, dequantize(q, s, z));
            }
        }
    }
}

/*
 * Straight-through estimator (named in Sec. 2.1, no formula given).  Reading:
 * the rounding is treated as the identity and the clamp as a hard gate, so
 *     dx = dy   where 0 <= u <= 2^b - 1   (u the rounded, unclamped code)
 *     dx = 0    elsewhere,
 * with scale and zero-point held constant (no gradient into the ranges).
 */
void granq_oracle_fakequant_bwd(const void *x, const void *dy, int dtype,
                                int64_t n, int64_t c, int64_t hw,
                                const float *scale, const float *zero_point,
                                int bits, void *dx)
{
    float qmax = code_max(bits);
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t ic = 0; ic < c; ++ic) {
            float s = scale[ic];
            float z = zero_point[ic];
            for (int64_t k = 0; k < hw; ++k) {
                int64_t i = (in * c + ic) * hw + k;
                float u = raw_code(load_elem(x, i, dtype), s, z);
                float g = load_elem(dy, i, dtype);
                if (!(u >= 0.0f && u <= qmax))
                    g = 0.0f;
                store_elem(dx, i, dtype, g);
            }
        }
    }
}

/*
 * The straight-through gate on its own, one bit per element: bit (i & 7) of byte
 * (i >> 3) is 1 where 0 <= u <= 2^b - 1 for the element with flat index i (u the
 * rounded, unclamped code of Eq. 1).  mask has (n*c*hw + 7) / 8 bytes; unused
 * high bits of the last byte are 0.
 */
void granq_oracle_gate_mask(const void *x, int dtype, int64_t n, int64_t c, int64_t hw,
                            const float *scale, const float *zero_point, int bits,
                            uint8_t *mask)
{
    float qmax = code_max(bits);
    int64_t total = n * c * hw;
    for (int64_t b = 0; b < (total + 7) / 8; ++b)
        mask[b] = 0;
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t ic = 0; ic < c; ++ic) {
            for (int64_t k = 0; k < hw; ++k) {
                int64_t i = (in * c + ic) * hw + k;
                float u = raw_code(load_elem(x, i, dtype), scale[ic], zero_point[ic]);
                if (u >= 0.0f && u <= qmax)
                    mask[i >> 3] |= (uint8_t)(1u << (i & 7));
            }
        }
    }
}

/* Backward from the gate bits: dx = dy where the bit is set, else 0. */
void granq_oracle_bwd_from_mask(const void *dy, const uint8_t *mask, int dtype,
                                int64_t total, void *dx)
{
    for (int64_t i = 0; i < total; ++i) {
        float g = load_elem(dy, i, dtype);
        if (!((mask[i >> 3] >> (i & 7)) & 1u))
            g = 0.0f;
        store_elem(dx, i, dtype, g);
    }
}

/*
 * Distortion of the fake-quantized tensor, the two figures of Table 2:
 *     cosine similarity  X.Q / (|X|_2 |Q|_2)     relative error  |X - Q|_2 / |X|_2
 * with Q = x_hat of the forward above.  Everything here is binary64: the
 * binary32 values are widened exactly, products, differences and sums are
 * doubles, summed in index order.
 * ch_sums[c][4] = { sum x*q, sum x^2, sum q^2, sum (x-q)^2 } per channel;
 * layer[0..3] = the same sums over all channels (added in channel order),
 * layer[4] = cosine similarity, layer[5] = relative error of the whole tensor.
 */
void granq_oracle_distortion(const void *x, int dtype, int64_t n, int64_t c, int64_t hw,
                             const float *scale, const float *zero_point, int bits,
                             double *ch_sums, double *layer)
{
    float qmax = code_max(bits);
    for (int64_t ic = 0; ic < c; ++ic) {
        double xq = 0.0, xx = 0.0, qq = 0.0, dd = 0.0;
        float s = scale[ic];
        float z = zero_point[ic];
        for (int64_t in = 0; in < n; ++in) {
            for (int64_t k = 0; k < hw; ++k) {
                float xf = load_elem(x, (in * c + ic) * hw + k, dtype);
                float qf = dequantize(clamp_code(raw_code(xf, s, z), qmax), s, z);
                double xd = (double)xf;
                double qd = (double)qf;
                double d = xd - qd;
                xq = xq + xd * qd;
                xx = xx + xd * xd;
                qq = qq + qd * qd;
                dd = dd + d * d;
            }
        }
        ch_sums[ic * 4 + 0] = xq;
        ch_sums[ic * 4 + 1] = xx;
        ch_sums[ic * 4 + 2] = qq;
        ch_sums[ic * 4 + 3] = dd;
    }
    for (int j = 0; j < 4; ++j) {
        double t = 0.0;
        for (int64_t ic = 0; ic < c; ++ic)
            t = t + ch_sums[ic * 4 + j];
        layer[j] = t;
    }
    layer[4] = layer[0] / (sqrt(layer[1]) * sqrt(layer[2]));
    layer[5] = sqrt(layer[3]) / sqrt(layer[1]);
}

/*
 * The two accumulation forms the paper contrasts, on a 1x1 weighted channel
 * sum with one weight per channel (fp32 storage only; accumulation in channel
 * order c = 0, 1, ...):
 *   in-loop scaling (Eq. 3):  y[n,k] = sum_c  w_c * s_c * (code[n,c,k] - z_c)
 *   pre-scaled (Eq. 6/Alg. 1): y[n,k] = sum_c  w_c * x_hat[n,c,k]
 * Eq. 3 is evaluated left to right: (w_c * s_c) * (code - z_c).
 */
void granq_oracle_accumulate_inloop(const uint8_t *codes,
                                    int64_t n, int64_t c, int64_t hw,
                                    const float *scale, const float *zero_point,
                                    const float *weight, float *y)
{
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t k = 0; k < hw; ++k) {
            float acc = 0.0f;
            for (int64_t ic = 0; ic < c; ++ic) {
                float d = (float)codes[(in * c + ic) * hw + k] - zero_point[ic];
                float ws = weight[ic] * scale[ic];
                float term = ws * d;
                acc = acc + term;
            }
            y[in * hw + k] = acc;
        }
    }
}

void granq_oracle_accumulate_prescaled(const float *x_hat,
                                       int64_t n, int64_t c, int64_t hw,
                                       const float *weight, float *y)
{
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t k = 0; k < hw; ++k) {
            float acc = 0.0f;
            for (int64_t ic = 0; ic < c; ++ic) {
                float term = weight[ic] * x_hat[(in * c + ic) * hw + k];
                acc = acc + term;
            }
            y[in * hw + k] = acc;
        }
    }
}

/*
 * Integer-domain accumulation (Eq. 3 with w_c * s_c folded into int8 weights).
 *
 * Fold: w'[o,c] = w[o,c] * s_c; the row is quantized symmetrically to int8 with
 * step a_o = max_c |w'[o,c]| / 127 (1 for an all-zero row):
 *     wq[o,c] = clamp(round(w'[o,c] / a_o), -127, 127),   corr[o] = sum_c wq[o,c] * z_c
 * (z_c is an integer held in a float).  binary32 operations, one rounding each; the
 * zero-point term is an exact integer sum, kept in 64 bits (|wq| <= 127, |z_c| < 2^24
 * and up to 65535 channels do not fit 32).
 */
void granq_oracle_fold_weights(const float *w, const float *scale, const float *zero_point,
                               int64_t o, int64_t c, int8_t *wq, int64_t *corr, float *out_scale)
{
    for (int64_t io = 0; io < o; ++io) {
        float amax = 0.0f;
        for (int64_t ic = 0; ic < c; ++ic) {
            float ws = w[io * c + ic] * scale[ic];
            if (fabsf(ws) > amax) amax = fabsf(ws);
        }
        float a = amax / 127.0f;
        if (!(a > 0.0f))
            a = 1.0f;
        int64_t cz = 0;
        for (int64_t ic = 0; ic < c; ++ic) {
            float ws = w[io * c + ic] * scale[ic];
            float q = rintf(ws / a);
            q = fminf(fmaxf(q, -127.0f), 127.0f);
            wq[io * c + ic] = (int8_t)q;
            cz += (int64_t)q * (int64_t)zero_point[ic];
        }
        corr[io] = cz;
        out_scale[io] = a;
    }
}

/*
 * The 1x1 convolution on the codes:
 *     y[n,o,k] = out_scale[o] * (float)( sum_c wq[o,c] * code[n,c,k]  -  corr[o] )
 * The integer expression is exact (64-bit); the conversion to float and the product round
 * once each.
 */
void granq_oracle_conv1x1_int8(const uint8_t *codes, int64_t n, int64_t c, int64_t hw, int64_t o,
                               const int8_t *wq, const int64_t *corr, const float *out_scale,
                               float *y)
{
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t io = 0; io < o; ++io) {
            for (int64_t k = 0; k < hw; ++k) {
                int64_t acc = 0;
                for (int64_t ic = 0; ic < c; ++ic)
                    acc += (int64_t)wq[io * c + ic] * (int64_t)codes[(in * c + ic) * hw + k];
                y[(in * o + io) * hw + k] = out_scale[io] * (float)(acc - corr[io]);
            }
        }
    }
}

/*
 * The accumulation of Eq. 6 with a full weight matrix: the 1x1 convolution over the
 * pre-scaled activations,
 *     y[n,o,k] = sum_c w[o,c] * x_hat[n,c,k],
 * in floating point.  This is the definition, summed in channel order in binary64: a product
 * of two binary32 (or 16-bit) values is exact in binary64, so only the additions round, each
 * to 2^-53.  w has x_hat's storage type, O rows of C.
 */
void granq_oracle_conv1x1_float(const void *x_hat, int dtype, int64_t n, int64_t c, int64_t hw,
                                int64_t o, const void *w, double *y)
{
    for (int64_t in = 0; in < n; ++in) {
        for (int64_t io = 0; io < o; ++io) {
            for (int64_t k = 0; k < hw; ++k) {
                double acc = 0.0;
                for (int64_t ic = 0; ic < c; ++ic) {
                    double wd = (double)load_elem(w, io * c + ic, dtype);
                    double xd = (double)load_elem(x_hat, (in * c + ic) * hw + k, dtype);
                    acc += wd * xd;
                }
                y[(in * o + io) * hw + k] = acc;
            }
        }
    }
}

/*
 * Codes of at most four bits, two per byte (the integer operands of Eq. 3 stored at their own
 * width): byte i holds the code q of Eq. 1 of the element with flat index 2i in its low
 * nibble and that of element 2i + 1 in its high nibble; an odd element count leaves the last
 * high nibble 0.  `codes` are the one-byte codes of the forward, each below 16.
 */
void granq_oracle_pack4(const uint8_t *codes, int64_t total, uint8_t *packed)
{
    for (int64_t i = 0; i < (total + 1) / 2; ++i) {
        uint8_t lo = codes[2 * i];
        uint8_t hi = 2 * i + 1 < total ? codes[2 * i + 1] : 0;
        packed[i] = (uint8_t)(lo | (hi << 4));
    }
}

/* The inverse: one byte per code again. */
void granq_oracle_unpack4(const uint8_t *packed, int64_t total, uint8_t *codes)
{
    for (int64_t i = 0; i < total; ++i) {
        uint8_t byte = packed[i / 2];
        codes[i] = (i % 2 == 0) ? (uint8_t)(byte & 0x0F) : (uint8_t)(byte >> 4);
    }
}
