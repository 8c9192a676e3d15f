// Stores of four neighbouring output pixels by the convolution kernels (a lane of those
// kernels owns four neighbouring pixels of one output channel).
#pragma once

#include "granq_device.h"

namespace granq {

// Four neighbouring output pixels to y at element index `at` (a multiple of 4; y aligned to
// four elements).
// STREAM: the output is large and will not be read again soon, so it is stored past the caches
// (non-temporal); an output that fits the memory-side cache is stored the ordinary way, which is
// faster there (1024 -> 256 channels at 14 x 14, batch 256, 51 MB of results: 28.8 against 35.3 us)
// and slower on large ones (256 -> 64 at 56 x 56, 205 MB: 87 against 66 us).
#ifndef GRANQ_CONV_STREAM_OUT_BYTES
#define GRANQ_CONV_STREAM_OUT_BYTES (96ll << 20)
#endif

// A kernel runs its epilogue as  if (stream_out) epilogue(Flag<true>{}); else epilogue(Flag<false>{});
// so that the choice is made once per wavefront.  The two copies differ only in the hint of
// their stores; the compiler folds stores of two branches that are otherwise identical into one
// and drops the hint, so the ordinary copy brackets itself with keep_apart().
template <bool B>
struct Flag {
    static constexpr bool value = B;
};
__device__ __forceinline__ void keep_apart() { asm volatile(""); }

template <typename OutT, bool STREAM>
__device__ __forceinline__ void store_pixels4(void *y, int64_t at, const f32x4 &v) {
    if constexpr (OutT::ESIZE == 4) {
        if constexpr (STREAM) __builtin_nontemporal_store(v, (f32x4 *)((float *)y + at));
        else *(f32x4 *)((float *)y + at) = v;
    } else {
        u32x2 w;
        w.x = OutT::pack2(v.x, v.y);
        w.y = OutT::pack2(v.z, v.w);
        if constexpr (STREAM) __builtin_nontemporal_store(w, (u32x2 *)((uint16_t *)y + at));
        else *(u32x2 *)((uint16_t *)y + at) = w;
    }
}

// The same when H*W is not a multiple of 4: a group's first pixel is then aligned to one element
// only, and a sample's last group has `valid` < 4 pixels.
template <typename OutT, bool STREAM>
__device__ __forceinline__ void store_pixels_ragged(void *y, int64_t at, const f32x4 &v, int valid) {
    typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
    typedef uint32_t u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));
    if (valid == 4) {
        if constexpr (OutT::ESIZE == 4) {
            if constexpr (STREAM) __builtin_nontemporal_store(v, (f32x4_a4 *)((float *)y + at));
            else *(f32x4_a4 *)((float *)y + at) = v;
        } else {
            u32x2 w;
            w.x = OutT::pack2(v.x, v.y);
            w.y = OutT::pack2(v.z, v.w);
            if constexpr (STREAM) __builtin_nontemporal_store(w, (u32x2_a2 *)((uint16_t *)y + at));
            else *(u32x2_a2 *)((uint16_t *)y + at) = w;
        }
    } else {
        OutT::store1(y, at, v.x);
        if (valid > 1) OutT::store1(y, at + 1, v.y);
        if (valid > 2) OutT::store1(y, at + 2, v.z);
    }
}

}  // namespace granq
