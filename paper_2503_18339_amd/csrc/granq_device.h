// Device-side building blocks shared by the GranQ kernels (gfx950, wave64).
//
// Everything here is arithmetic-exact plumbing: 128-bit loads and stores,
// bfloat16 widening / narrowing, wavefront and block min/max reductions, and the
// three lines of arithmetic that define the quantizer (Eq. 1, Eq. 6 of the paper
// and the straight-through gate).  The arithmetic is written so that the
// compiler emits one correctly rounded IEEE binary32 operation per source
// operation (the build passes -ffp-contract=off; HIP's default float division
// is the correctly rounded one).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace granq {

#ifndef GRANQ_BLOCK
#define GRANQ_BLOCK 256
#endif
constexpr int kBlock = GRANQ_BLOCK;   // threads per block: four wavefronts
constexpr int kWave = 64;     // CDNA wavefront width

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// storage traits: one 16-byte vector per lane and per load
// ---------------------------------------------------------------------------

struct F32 {
    using vec_t = f32x4;            // 4 floats
    using code_t = uint32_t;        // 4 packed 8-bit codes
    static constexpr int VEC = 4;
    static constexpr int ESIZE = 4;
    __device__ static inline void unpack(const vec_t &v, float (&f)[VEC]) {
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static inline vec_t pack(const float (&f)[VEC]) {
        vec_t v; v.x = f[0]; v.y = f[1]; v.z = f[2]; v.w = f[3];
        return v;
    }
    __device__ static inline code_t pack_codes(const float (&q)[VEC]) {
        return (uint32_t)q[0] | ((uint32_t)q[1] << 8) | ((uint32_t)q[2] << 16) | ((uint32_t)q[3] << 24);
    }
    // codes below 16, two per byte, element i in nibble i
    using code4_t = uint16_t;
    __device__ static inline code4_t pack_codes4(const float (&q)[VEC]) {
        return (uint16_t)((uint32_t)q[0] | ((uint32_t)q[1] << 4) | ((uint32_t)q[2] << 8) | ((uint32_t)q[3] << 12));
    }
    // keep element i of g where keep[i], else +0
    __device__ static inline vec_t gate(const vec_t &g, const bool (&keep)[VEC]) {
        vec_t r;
        r.x = keep[0] ? g.x : 0.0f; r.y = keep[1] ? g.y : 0.0f;
        r.z = keep[2] ? g.z : 0.0f; r.w = keep[3] ? g.w : 0.0f;
        return r;
    }
    __device__ static inline float load1(const void *p, int64_t i) { return ((const float *)p)[i]; }
    __device__ static inline void store1(void *p, int64_t i, float v) { ((float *)p)[i] = v; }
    __device__ static inline void store_gated1(void *dx, const void *dy, int64_t i, bool keep) {
        ((float *)dx)[i] = keep ? ((const float *)dy)[i] : 0.0f;
    }
};

// bfloat16 -> binary32 is exact: the 16 bits become the high half of the word.
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// binary32 -> bfloat16, round to nearest even, finite inputs: add 0x7FFF plus
// the lowest kept bit, then drop the low half.
__device__ inline uint32_t bf16_round(float f) {
    uint32_t b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// What the two 16-bit storage types share: eight elements in four 32-bit words,
// element 2i in the low half of word i.
struct Pack16 {
    using vec_t = u32x4;            // 8 elements in four 32-bit words
    using code_t = u32x2;           // 8 packed 8-bit codes
    static constexpr int VEC = 8;
    static constexpr int ESIZE = 2;
    __device__ static inline code_t pack_codes(const float (&q)[VEC]) {
        code_t c;
        c.x = (uint32_t)q[0] | ((uint32_t)q[1] << 8) | ((uint32_t)q[2] << 16) | ((uint32_t)q[3] << 24);
        c.y = (uint32_t)q[4] | ((uint32_t)q[5] << 8) | ((uint32_t)q[6] << 16) | ((uint32_t)q[7] << 24);
        return c;
    }
    using code4_t = uint32_t;       // 8 packed 4-bit codes, element i in nibble i
    __device__ static inline code4_t pack_codes4(const float (&q)[VEC]) {
        uint32_t c = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) c |= (uint32_t)q[e] << (4 * e);
        return c;
    }
    __device__ static inline vec_t gate(const vec_t &g, const bool (&keep)[VEC]) {
        vec_t r;
        r.x = g.x & ((keep[0] ? 0x0000FFFFu : 0u) | (keep[1] ? 0xFFFF0000u : 0u));
        r.y = g.y & ((keep[2] ? 0x0000FFFFu : 0u) | (keep[3] ? 0xFFFF0000u : 0u));
        r.z = g.z & ((keep[4] ? 0x0000FFFFu : 0u) | (keep[5] ? 0xFFFF0000u : 0u));
        r.w = g.w & ((keep[6] ? 0x0000FFFFu : 0u) | (keep[7] ? 0xFFFF0000u : 0u));
        return r;
    }
    __device__ static inline void store_gated1(void *dx, const void *dy, int64_t i, bool keep) {
        ((uint16_t *)dx)[i] = keep ? ((const uint16_t *)dy)[i] : (uint16_t)0;
    }
};

struct BF16 : Pack16 {
    __device__ static inline void unpack(const vec_t &v, float (&f)[VEC]) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
    // v_cvt_pk_bf16_f32 rounds to nearest even; checked against bf16_round on every
    // finite binary32 pattern, subnormals included.
    __device__ static inline uint32_t pack2(float lo, float hi) {
        f32x2 v = {lo, hi};
        bf16x2 b = __builtin_convertvector(v, bf16x2);
        uint32_t u;
        __builtin_memcpy(&u, &b, sizeof u);
        return u;
    }
    __device__ static inline vec_t pack(const float (&f)[VEC]) {
        vec_t v;
        v.x = pack2(f[0], f[1]);
        v.y = pack2(f[2], f[3]);
        v.z = pack2(f[4], f[5]);
        v.w = pack2(f[6], f[7]);
        return v;
    }
    __device__ static inline float load1(const void *p, int64_t i) {
        return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
    }
    __device__ static inline void store1(void *p, int64_t i, float v) {
        ((uint16_t *)p)[i] = (uint16_t)bf16_round(v);
    }
};

// IEEE binary16.  Widening (v_cvt_f32_f16) is exact, subnormals included; narrowing
// (v_cvt_f16_f32) rounds to nearest even in the default rounding mode, produces
// subnormals and overflows to infinity above 65504 + half a step.
struct F16 : Pack16 {
    // The value to narrow is a binary32 result that must be rounded to binary32 first and to
    // binary16 second.  Left alone, the compiler fuses the multiply that produced it with the
    // narrowing (v_fma_mixlo_f16), which rounds once, from the exact product: a different
    // binary16 value whenever the binary32 rounding lands exactly between two binary16 values.
    // The empty statement pins the binary32 value in a register.
    __device__ static inline float rounded_f32(float v) {
        asm volatile("" : "+v"(v));
        return v;
    }
    __device__ static inline void unpack2(uint32_t w, float &lo, float &hi) {
        f16x2 h;
        __builtin_memcpy(&h, &w, sizeof h);
        f32x2 v = __builtin_convertvector(h, f32x2);
        lo = v.x;
        hi = v.y;
    }
    __device__ static inline void unpack(const vec_t &v, float (&f)[VEC]) {
        unpack2(v.x, f[0], f[1]);
        unpack2(v.y, f[2], f[3]);
        unpack2(v.z, f[4], f[5]);
        unpack2(v.w, f[6], f[7]);
    }
    __device__ static inline uint32_t pack2(float lo, float hi) {
        f32x2 v = {rounded_f32(lo), rounded_f32(hi)};
        f16x2 h = __builtin_convertvector(v, f16x2);
        uint32_t u;
        __builtin_memcpy(&u, &h, sizeof u);
        return u;
    }
    __device__ static inline vec_t pack(const float (&f)[VEC]) {
        vec_t v;
        v.x = pack2(f[0], f[1]);
        v.y = pack2(f[2], f[3]);
        v.z = pack2(f[4], f[5]);
        v.w = pack2(f[6], f[7]);
        return v;
    }
    __device__ static inline float load1(const void *p, int64_t i) {
        return (float)((const _Float16 *)p)[i];
    }
    __device__ static inline void store1(void *p, int64_t i, float v) {
        ((_Float16 *)p)[i] = (_Float16)rounded_f32(v);
    }
};

// ---------------------------------------------------------------------------
// the quantizer's arithmetic
// ---------------------------------------------------------------------------

// Eq. 1 without the clamp: round_half_even(x / s + z).  v_rndne_f32 rounds
// ties to even.
__device__ inline float raw_code(float x, float s, float z) {
    float t = x / s;
    float v = t + z;
    return __builtin_rintf(v);
}

// Clamp to [0, qmax]: the median of (u, 0, qmax), one instruction.
__device__ inline float clamp_code(float u, float qmax) {
    return __builtin_amdgcn_fmed3f(u, 0.0f, qmax);
}

// Dequantization of Eq. 6: s * (q - z).
__device__ inline float dequant(float q, float s, float z) {
    float d = q - z;
    return s * d;
}

// Straight-through gate: the clamp was inactive.
__device__ inline bool in_range(float u, float qmax) { return u >= 0.0f && u <= qmax; }

// ---------------------------------------------------------------------------
// wavefront / block min-max
// ---------------------------------------------------------------------------

template <int CTRL>
__device__ inline float dpp_move(float v) {
    int i = __float_as_int(v);
    return __int_as_float(__builtin_amdgcn_update_dpp(i, i, CTRL, 0xF, 0xF, false));
}

// DPP controls: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror,
// row_mirror.  After the four steps every lane of a 16-lane row holds the row's
// result; the four rows are then combined through scalar registers.
constexpr int kDppQuadSwap1 = 0xB1;
constexpr int kDppQuadSwap2 = 0x4E;
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

__device__ inline float readlane_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Minimum over the 64 lanes of the wavefront, returned in every lane.
__device__ inline float wave_min(float v) {
    v = __builtin_fminf(v, dpp_move<kDppQuadSwap1>(v));
    v = __builtin_fminf(v, dpp_move<kDppQuadSwap2>(v));
    v = __builtin_fminf(v, dpp_move<kDppRowHalfMirror>(v));
    v = __builtin_fminf(v, dpp_move<kDppRowMirror>(v));
    float a = __builtin_fminf(readlane_f(v, 0), readlane_f(v, 16));
    float b = __builtin_fminf(readlane_f(v, 32), readlane_f(v, 48));
    return __builtin_fminf(a, b);
}

__device__ inline float wave_max(float v) {
    v = __builtin_fmaxf(v, dpp_move<kDppQuadSwap1>(v));
    v = __builtin_fmaxf(v, dpp_move<kDppQuadSwap2>(v));
    v = __builtin_fmaxf(v, dpp_move<kDppRowHalfMirror>(v));
    v = __builtin_fmaxf(v, dpp_move<kDppRowMirror>(v));
    float a = __builtin_fmaxf(readlane_f(v, 0), readlane_f(v, 16));
    float b = __builtin_fmaxf(readlane_f(v, 32), readlane_f(v, 48));
    return __builtin_fmaxf(a, b);
}

// Order-preserving map float -> uint32 (for non-NaN values a < b  <=>  key(a) <
// key(b), with -0 just below +0), so that LDS integer atomics can take minima
// and maxima of floats.  Min and max are exact, hence independent of the order
// in which lanes arrive.
__device__ inline uint32_t float_key(float f) {
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}
constexpr uint32_t kKeyPosInf = 0xFF800000u;   // float_key(+inf): identity of min
constexpr uint32_t kKeyNegInf = 0x007FFFFFu;   // float_key(-inf): identity of max

}  // namespace granq
