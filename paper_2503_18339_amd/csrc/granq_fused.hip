// Alg. 1 of the paper up to the accumulation in ONE call: ranges (Eq. 4), scale and
// zero-point (Eq. 5), quantize-clamp-dequantize (Eq. 1, 6).
//
// Small activations -- the paper's own latency table is taken at batch 16 on CIFAR-size
// feature maps, where a channel holds a few thousand elements -- are bound by the cost of
// each dependent launch, not by memory.  For them one block owns one channel from start to
// finish: it loads the channel into registers, reduces min / max across the block, computes
// the two parameters and quantizes what it holds.  One launch instead of three, one read of
// x.  Larger tensors take granq_calibrate followed by granq_fakequant_fwd.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_plan.h"
#include "granq_block.h"
#include "granq_internal.h"

namespace granq {

// One block of kFusedBlock threads owns a channel and keeps all of it in registers between
// the min / max sweep and the quantization: kFusedVecs 16-byte vectors per thread, or
// kFusedScalars single elements where the shape or the pointers rule out 16-byte accesses.
constexpr int kFusedBlock = 1024;
constexpr int kFusedVecs = 8;
constexpr int kFusedScalars = 32;
// Largest tensor (bytes) handled by one block per channel when the two-launch form is also possible.
#ifndef GRANQ_ONE_BLOCK_MAX_BYTES
#define GRANQ_ONE_BLOCK_MAX_BYTES ((int64_t)8 << 20)
#endif

// Block-wide min and max over kFusedBlock threads, result in every thread.
__device__ inline void fused_block_minmax(float &mn, float &mx, float (*part)[kFusedBlock / kWave]) {
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
    for (int w = 1; w < kFusedBlock / kWave; ++w) {
        mn = __builtin_fminf(mn, part[0][w]);
        mx = __builtin_fmaxf(mx, part[1][w]);
    }
}

// Block ic: channel ic = n slabs of hw consecutive elements, slab `in` at (in * c + ic) * hw.
// VECTOR: units are 16-byte vectors (hw a multiple of T::VEC, pointers 16-byte aligned), else
// single elements; `units` = units in the channel, `slab_div` divides by the units per slab.
template <typename T, bool VECTOR>
__global__ __launch_bounds__(kFusedBlock) void fq_channel_block(
    const void *x, void *x_hat, uint8_t *__restrict__ codes,
    float *__restrict__ ch_min, float *__restrict__ ch_max, float *__restrict__ scale,
    float *__restrict__ zero_point, float qmax, uint32_t units, int64_t c, FastDiv slab_div)
{
    constexpr int PER = VECTOR ? kFusedVecs : kFusedScalars;
    constexpr int VEC = T::VEC;
    using vec_t = typename T::vec_t;
    __shared__ float part[2][kFusedBlock / kWave];
    const int64_t ic = blockIdx.x;
    const uint32_t per_slab = slab_div.d;

    int64_t at[PER];                                    // unit index in the tensor, -1: none
    vec_t vin[VECTOR ? PER : 1];
    float fin[VECTOR ? 1 : PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const uint32_t u = threadIdx.x + i * kFusedBlock;
        at[i] = -1;
        if (u < units) {
            const uint32_t in = fastdiv(u, slab_div);
            at[i] = ((int64_t)in * c + ic) * per_slab + (u - in * per_slab);
        }
    }
#pragma unroll
    for (int i = 0; i < PER; ++i)                       // all loads in flight together
        if (at[i] >= 0) {
            if (VECTOR) vin[VECTOR ? i : 0] = ((const vec_t *)x)[at[i]];
            else fin[VECTOR ? 0 : i] = T::load1(x, at[i]);
        }
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < PER; ++i)
        if (at[i] >= 0) {
            if (VECTOR) {
                float f[VEC];
                T::unpack(vin[VECTOR ? i : 0], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    mn = __builtin_fminf(mn, f[e]);
                    mx = __builtin_fmaxf(mx, f[e]);
                }
            } else {
                mn = __builtin_fminf(mn, fin[VECTOR ? 0 : i]);
                mx = __builtin_fmaxf(mx, fin[VECTOR ? 0 : i]);
            }
        }
    fused_block_minmax(mn, mx, part);

    float s, z;
    channel_scale(mn, mx, qmax, s, z);
    if (threadIdx.x == 0) {
        ch_min[ic] = mn;
        ch_max[ic] = mx;
        scale[ic] = s;
        zero_point[ic] = z;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i)
        if (at[i] >= 0) {
            if (VECTOR) {
                float f[VEC], q[VEC];
                T::unpack(vin[VECTOR ? i : 0], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    q[e] = clamp_code(raw_code(f[e], s, z), qmax);
                    f[e] = dequant(q[e], s, z);
                }
                if (x_hat) ((vec_t *)x_hat)[at[i]] = T::pack(f);
                if (codes) ((typename T::code_t *)codes)[at[i]] = T::pack_codes(q);
            } else {
                const float q = clamp_code(raw_code(fin[VECTOR ? 0 : i], s, z), qmax);
                if (x_hat) T::store1(x_hat, at[i], dequant(q, s, z));
                if (codes) codes[at[i]] = (uint8_t)q;
            }
        }
}

template <typename T>
static void launch_channel_block(bool vector, const void *x, void *x_hat, uint8_t *codes, float *ch_min,
                                 float *ch_max, float *scale, float *zero_point, float qmax, uint32_t units,
                                 int64_t c, FastDiv slab_div, hipStream_t hs) {
    dim3 grid((uint32_t)c), block(kFusedBlock);
    if (vector)
        launch_kernel((fq_channel_block<T, true>), grid, block, 0, hs, x, x_hat, codes, ch_min, ch_max, scale,
                           zero_point, qmax, units, c, slab_div);
    else
        launch_kernel((fq_channel_block<T, false>), grid, block, 0, hs, x, x_hat, codes, ch_min, ch_max, scale,
                           zero_point, qmax, units, c, slab_div);
}

// How granq_calibrate_fakequant_fwd handles a tensor: one block per channel (one launch) when
// the channel fits a block's registers and the tensor is small, else the two-launch form where
// it applies, else granq_calibrate + granq_fakequant_fwd (three launches).
struct OneCallChoice {
    int launches;        // 1, 2 or 3
    bool vector;         // one launch: 16-byte units
    int64_t units;       // one launch: units per channel
};

static OneCallChoice one_call_choice(const granq_desc_t *desc, const void *x, const void *x_hat,
                                     const uint8_t *codes_or_null) {
    OneCallChoice ch{3, false, 0};
    const int64_t hw = desc->h > 0 && desc->w > 0 ? desc->h * desc->w : 0;
    const bool known = desc->dtype == GRANQ_F32 || desc->dtype == GRANQ_BF16 || desc->dtype == GRANQ_F16;
    const int esize = desc->dtype == GRANQ_F32 ? 4 : 2;
    const int vec = 16 / esize;
    const bool sane = known && desc->n > 0 && desc->c > 0 && hw > 0 && desc->c < ((int64_t)1 << 31) &&
                      hw <= ((int64_t)1 << 20) && desc->n <= ((int64_t)1 << 20);
    if (!sane) return ch;
    ch.vector = hw % vec == 0 && ((uintptr_t)x & 15u) == 0 && ((uintptr_t)x_hat & 15u) == 0 &&
                ((uintptr_t)codes_or_null % (uintptr_t)vec) == 0;
    ch.units = ch.vector ? desc->n * (hw / vec) : desc->n * hw;
    const bool fits = ch.units <= (int64_t)kFusedBlock * (ch.vector ? kFusedVecs : kFusedScalars);
    const bool two = two_launches_apply(x, desc, x_hat, codes_or_null);
    // C blocks are a good use of the chip only while the tensor is small; beyond that the
    // two-launch form (all compute units on the reduction, then on the forward) wins
    const int64_t bytes = desc->n * desc->c * hw * esize;
    if (fits && (bytes <= GRANQ_ONE_BLOCK_MAX_BYTES || !two)) ch.launches = 1;
    else ch.launches = two ? 2 : 3;
    return ch;
}

int one_call_forward_launches(const granq_desc_t *desc) {
    return one_call_choice(desc, (const void *)256, (const void *)256, nullptr).launches;
}

}  // namespace granq

using namespace granq;

extern "C" {

granq_status_t granq_calibrate_fakequant_fwd(const void *x, const granq_desc_t *desc, int bits,
                                             float *ch_min, float *ch_max, float *scale,
                                             float *zero_point, void *x_hat, uint8_t *codes_or_null,
                                             void *workspace, size_t workspace_bytes, void *stream) {
    if (!desc) return GRANQ_ERR_INVALID_ARG;
    const int64_t hw = desc->h > 0 && desc->w > 0 ? desc->h * desc->w : 0;
    const bool known = desc->dtype == GRANQ_F32 || desc->dtype == GRANQ_BF16 || desc->dtype == GRANQ_F16;
    const int esize = desc->dtype == GRANQ_F32 ? 4 : 2;
    const int vec = 16 / esize;
    // what only the forward would refuse is refused before anything is launched
    if (!x_hat && !codes_or_null) return GRANQ_ERR_INVALID_ARG;
    if (known && ((uintptr_t)x_hat & ((uintptr_t)esize - 1))) return GRANQ_ERR_UNSUPPORTED;

    const OneCallChoice choice = one_call_choice(desc, x, x_hat, codes_or_null);
    if (choice.launches == 2)
        return calibrate_fwd_two_launches(x, desc, bits, ch_min, ch_max, scale, zero_point, x_hat,
                                          codes_or_null, workspace, workspace_bytes, stream);
    if (choice.launches == 3) {
        // every check of the two calls applies
        granq_status_t st = granq_calibrate(x, desc, bits, ch_min, ch_max, scale, zero_point, workspace,
                                            workspace_bytes, stream);
        if (st != GRANQ_OK) return st;
        return granq_fakequant_fwd(x, desc, scale, zero_point, bits, x_hat, codes_or_null, stream);
    }
    const bool vector = choice.vector;
    const int64_t units = choice.units;
    // the same argument checks as the two calls make
    if (!x || !ch_min || !ch_max || !scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (((uintptr_t)x & ((uintptr_t)esize - 1)) || ((uintptr_t)ch_min & 3u) || ((uintptr_t)ch_max & 3u) ||
        ((uintptr_t)scale & 3u) || ((uintptr_t)zero_point & 3u))
        return GRANQ_ERR_UNSUPPORTED;
    size_t need = 0;
    granq_status_t st = granq_workspace_bytes(desc, &need);
    if (st != GRANQ_OK) return st;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u)) return GRANQ_ERR_WORKSPACE;

    const float qmax = (float)((1 << bits) - 1);
    const FastDiv slab_div = make_fastdiv((uint32_t)(vector ? hw / vec : hw));
    hipStream_t hs = (hipStream_t)stream;
    if (desc->dtype == GRANQ_F32)
        launch_channel_block<F32>(vector, x, x_hat, codes_or_null, ch_min, ch_max, scale, zero_point, qmax,
                                  (uint32_t)units, desc->c, slab_div, hs);
    else if (desc->dtype == GRANQ_BF16)
        launch_channel_block<BF16>(vector, x, x_hat, codes_or_null, ch_min, ch_max, scale, zero_point, qmax,
                                   (uint32_t)units, desc->c, slab_div, hs);
    else
        launch_channel_block<F16>(vector, x, x_hat, codes_or_null, ch_min, ch_max, scale, zero_point, qmax,
                                  (uint32_t)units, desc->c, slab_div, hs);
    return launched();
}

}  // extern "C"
