// Block-level helpers of the kernels in which one block owns one channel (or row) from
// start to finish.
#pragma once

#include <float.h>
#include <stdint.h>

#include "granq_device.h"

namespace granq {

// Block-wide min and max, result in every thread.  `part` is LDS scratch of the caller;
// a second call needs a __syncthreads() before it reuses the same scratch.
__device__ inline void block_minmax(float &mn, float &mx, float (*part)[kBlock / kWave]) {
    mn = wave_min(mn);
    mx = wave_max(mx);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        part[0][wave] = mn;
        part[1][wave] = mx;
    }
    __syncthreads();
    mn = part[0][0];
    mx = part[1][0];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) {
        mn = __builtin_fminf(mn, part[0][w]);
        mx = __builtin_fmaxf(mx, part[1][w]);
    }
}

// Eq. 2 / Eq. 5 for one channel, with the degenerate-range rule: a scale that comes out zero,
// subnormal or NaN becomes 1; a zero-point of -0 becomes +0.
__device__ inline void channel_scale(float mn, float mx, float qmax, float &s, float &z) {
    const float range = mx - mn;
    s = range / qmax;
    if (!(s >= FLT_MIN)) s = 1.0f;
    z = __builtin_rintf((-mn) / s) + 0.0f;
}

}  // namespace granq
