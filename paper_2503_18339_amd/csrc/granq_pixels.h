// Stores of four neighbouring output pixels by the convolution kernels (a lane of those
// kernels owns four neighbouring pixels of one output channel).
#pragma once

#include "granq_device.h"

namespace granq {

// Four neighbouring output pixels to y at element index `at` (a multiple of 4; y aligned to
// four elements).
template <typename OutT>
__device__ __forceinline__ void store_pixels4(void *y, int64_t at, const f32x4 &v) {
    if constexpr (OutT::ESIZE == 4) {
        __builtin_nontemporal_store(v, (f32x4 *)((float *)y + at));
    } else {
        u32x2 w;
        w.x = OutT::pack2(v.x, v.y);
        w.y = OutT::pack2(v.z, v.w);
        __builtin_nontemporal_store(w, (u32x2 *)((uint16_t *)y + at));
    }
}

// The same when H*W is not a multiple of 4: a group's first pixel is then aligned to one element
// only, and a sample's last group has `valid` < 4 pixels.
template <typename OutT>
__device__ __forceinline__ void store_pixels_ragged(void *y, int64_t at, const f32x4 &v, int valid) {
    typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
    typedef uint32_t u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));
    if (valid == 4) {
        if constexpr (OutT::ESIZE == 4) {
            __builtin_nontemporal_store(v, (f32x4_a4 *)((float *)y + at));
        } else {
            u32x2 w;
            w.x = OutT::pack2(v.x, v.y);
            w.y = OutT::pack2(v.z, v.w);
            __builtin_nontemporal_store(w, (u32x2_a2 *)((uint16_t *)y + at));
        }
    } else {
        OutT::store1(y, at, v.x);
        if (valid > 1) OutT::store1(y, at + 1, v.y);
        if (valid > 2) OutT::store1(y, at + 2, v.z);
    }
}

}  // namespace granq
