// Correctly rounded binary32 quotient x / s with a per-channel reciprocal.
//
// Eq. 1 of the paper divides every element by its channel's scale.  A general
// IEEE division costs eleven instructions on CDNA; here the divisor is shared
// by all elements of a channel, so its correctly rounded reciprocal
// r = RN(1/s) is computed once (by a true division) and each element costs
// five:
//
//     q0 = RN(x * r)                      within 2 ulp of x/s
//     e0 = x - s*q0      (one FMA, exact)
//     q1 = RN(q0 + e0*r)                  within 1 ulp of x/s
//     e1 = x - s*q1      (one FMA, exact)
//     q  = RN(q1 + e1*r)                  = RN(x/s)
//
// The last step is Markstein's theorem (P. Markstein, "Computation of
// elementary functions on the IBM RISC System/6000 processor", 1990; also
// Muller et al., Handbook of Floating-Point Arithmetic, "division with an FMA"):
// with r the correctly rounded reciprocal, q1 within one ulp of the quotient and
// the residual exact, the corrected quotient is the correctly rounded one.  It
// needs the absence of overflow and underflow in the intermediates, which the
// caller guarantees by taking this path only when
//
//     2^-30 <= s <= 2^60   and   |z| <= 2^26          (quotient_fast_ok)
//
// and by clamping x to +-2^90 first (quotient_clamp).  Why that is enough, for
// the use made of the quotient, u = round(x/s + z) clamped to [0, 2^b - 1]:
//   - |x| >= 2^-100 and |x/s| >= 2^-40: every intermediate is a normal number,
//     the residuals are exact, the theorem applies: q is bit-identical to x / s.
//   - otherwise the true quotient is below 2^-40 in magnitude and the computed
//     one below 2^-29 (a product or residual may have underflowed); adding
//     either to z gives z itself, or something below 1/2 when z is small, so u
//     is the same.
//   - |x| >  2^90: true and clamped quotient both exceed 2^30 > |z| + 2^b in
//     magnitude with the sign of x, so u is clamped to the same end and the
//     straight-through gate is closed either way.
// Channels outside the window use the ordinary division.
//
// This header is plain C++ so that the same function can be compiled for the
// host and checked against `/` there.
#pragma once

#if defined(__HIPCC__)
#define GRANQ_HD __host__ __device__
#else
#define GRANQ_HD
#endif

namespace granq {

GRANQ_HD inline bool quotient_fast_ok(float s, float z) {
    // written so that NaN fails every test
    return s >= 0x1p-30f && s <= 0x1p60f && z >= -0x1p26f && z <= 0x1p26f;
}

GRANQ_HD inline float quotient_clamp(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(x, -0x1p90f, 0x1p90f);   // median of three: one instruction
#else
    return __builtin_fminf(__builtin_fmaxf(x, -0x1p90f), 0x1p90f);
#endif
}

// x already clamped; r == 1.0f / s (correctly rounded).
GRANQ_HD inline float quotient_fast(float x, float s, float r) {
    float q0 = x * r;
    float e0 = __builtin_fmaf(-s, q0, x);
    float q1 = __builtin_fmaf(e0, r, q0);
    float e1 = __builtin_fmaf(-s, q1, x);
    return __builtin_fmaf(e1, r, q1);
}

}  // namespace granq
