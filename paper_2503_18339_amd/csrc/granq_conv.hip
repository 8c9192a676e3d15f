// Integer-domain accumulation on the matrix cores: the 1x1 convolution that
// consumes the quantized activations, from their integer codes (Eq. 3 of the
// paper with w_c * s_c folded into int8 weights and the zero-point term summed
// once per output channel).
//
// Per sample the product is  D[O x HW] = Wq[O x C] . code[C x HW], int8 x int8 ->
// int32 with v_mfma_i32_32x32x16_i8.  A wavefront owns 128 consecutive pixels and
// all output channels.  Operand layout of the instruction (64 lanes, lane l):
//   A (32 x 16): row l % 32, eight consecutive k starting at 8 * (l / 32), one byte each
//   B (16 x 32): column l % 32, the same eight k
//   D (32 x 32): column l % 32, register r holds row 8 * (r / 4) + 4 * (l / 32) + r % 4
// The codes are NCHW, so consecutive k (channels) of one pixel are H*W bytes
// apart: a lane loads, for its eight channels, one dword (four neighbouring
// pixels) each and transposes the 8 x 4 bytes in registers into four B operands;
// MFMA j of a group therefore covers pixels 4 * (l % 32) + j, and a lane ends up
// with four neighbouring pixels of every output row: one 16-byte store per row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"

namespace granq {

typedef int i32x16 __attribute__((ext_vector_type(16)));

// OT = output-channel tiles of 32 handled by one wavefront.
template <int OT>
__global__ __launch_bounds__(kBlock) void conv1x1_i8_mfma(
    const uint8_t *__restrict__ codes, const int8_t *__restrict__ wq, const int32_t *__restrict__ corr,
    const float *__restrict__ out_scale, float *__restrict__ y, int64_t c, int64_t hw, int64_t o,
    int64_t o_base)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int half = lane / 32, col = lane % 32;
    const int64_t n = blockIdx.y;
    const int64_t pb = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * 128 + 4 * col;
    const bool live = pb < hw;                         // hw % 4 == 0: a lane's four pixels are all in or all out

    i32x16 acc[OT][4];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][j][r] = 0;

    const uint8_t *src = codes + (n * c + 8 * half) * hw + (live ? pb : 0);
    for (int64_t k0 = 0; k0 < c; k0 += 16) {
        uint32_t d[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) d[i] = live ? *(const uint32_t *)(src + (k0 + i) * hw) : 0u;
        long b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {                  // byte j of each of the eight dwords
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= ((d[i] >> (8 * j)) & 0xFFu) << (8 * i);
                hi |= ((d[4 + i] >> (8 * j)) & 0xFFu) << (8 * i);
            }
            b[j] = (long)(((uint64_t)hi << 32) | lo);
        }
#pragma unroll
        for (int t = 0; t < OT; ++t) {
            const long a = *(const long *)(wq + (o_base + 32 * t + col) * c + k0 + 8 * half);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[t][j] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a, b[j], acc[t][j], 0, 0, 0);
        }
    }
    if (!live) return;
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t oc = o_base + 32 * t + 8 * (r / 4) + 4 * half + (r % 4);
            const int32_t cz = corr[oc];
            const float a = out_scale[oc];
            f32x4 v;
            v.x = a * (float)(acc[t][0][r] - cz);
            v.y = a * (float)(acc[t][1][r] - cz);
            v.z = a * (float)(acc[t][2][r] - cz);
            v.w = a * (float)(acc[t][3][r] - cz);
            __builtin_nontemporal_store(v, (f32x4 *)(y + (n * o + oc) * hw + pb));
        }
}

// Any shape: one thread per output element, integer loop over the channels.
__global__ __launch_bounds__(kBlock) void conv1x1_i8_plain(
    const uint8_t *__restrict__ codes, const int8_t *__restrict__ wq, const int32_t *__restrict__ corr,
    const float *__restrict__ out_scale, float *__restrict__ y, int64_t c, int64_t hw, int64_t o)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t oc = blockIdx.y;
    const int64_t n = blockIdx.z;
    if (k >= hw) return;
    int32_t acc = 0;
    for (int64_t ic = 0; ic < c; ++ic)
        acc += (int32_t)wq[oc * c + ic] * (int32_t)codes[(n * c + ic) * hw + k];
    y[(n * o + oc) * hw + k] = out_scale[oc] * (float)(acc - corr[oc]);
}

// One block per output channel: fold the activation scale into the weights and
// quantize the row to int8 (symmetric), sum the zero-point term.
__global__ __launch_bounds__(kBlock) void fold_weights_kernel(
    const float *__restrict__ w, const float *__restrict__ scale, const float *__restrict__ zero_point,
    int64_t c, int8_t *__restrict__ wq, int32_t *__restrict__ corr, float *__restrict__ out_scale)
{
    __shared__ float part[kBlock / kWave];
    __shared__ int32_t ipart[kBlock / kWave];
    const int64_t oc = blockIdx.x;
    float amax = 0.0f;
    for (int64_t ic = threadIdx.x; ic < c; ic += kBlock) {
        const float ws = w[oc * c + ic] * scale[ic];
        amax = __builtin_fmaxf(amax, __builtin_fabsf(ws));
    }
    amax = wave_max(amax);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = amax;
    __syncthreads();
    amax = part[0];
    for (int i = 1; i < kBlock / kWave; ++i) amax = __builtin_fmaxf(amax, part[i]);
    float a = amax / 127.0f;
    if (!(a > 0.0f)) a = 1.0f;
    int32_t cz = 0;
    for (int64_t ic = threadIdx.x; ic < c; ic += kBlock) {
        const float ws = w[oc * c + ic] * scale[ic];
        float q = __builtin_rintf(ws / a);
        q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
        const int32_t qi = (int32_t)q;
        wq[oc * c + ic] = (int8_t)qi;
        cz += qi * (int32_t)zero_point[ic];
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) cz += __shfl_xor(cz, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) ipart[threadIdx.x / kWave] = cz;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t t = 0;
        for (int i = 0; i < kBlock / kWave; ++i) t += ipart[i];
        corr[oc] = t;
        out_scale[oc] = a;
    }
}

}  // namespace granq

using namespace granq;

extern "C" {

granq_status_t granq_fold_weights(const float *w, const float *scale, const float *zero_point,
                                  int64_t o, int64_t c, int8_t *wq, int32_t *corr, float *out_scale,
                                  void *stream) {
    if (!w || !scale || !zero_point || !wq || !corr || !out_scale) return GRANQ_ERR_INVALID_ARG;
    if (o <= 0 || c <= 0) return GRANQ_ERR_INVALID_ARG;
    if (o >= ((int64_t)1 << 31) || c >= ((int64_t)1 << 24)) return GRANQ_ERR_UNSUPPORTED;
    if (((uintptr_t)w & 3u) || ((uintptr_t)scale & 3u) || ((uintptr_t)zero_point & 3u) ||
        ((uintptr_t)corr & 3u) || ((uintptr_t)out_scale & 3u))
        return GRANQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fold_weights_kernel, dim3((uint32_t)o), dim3(kBlock), 0, (hipStream_t)stream,
                       w, scale, zero_point, c, wq, corr, out_scale);
    return hipGetLastError() == hipSuccess ? GRANQ_OK : GRANQ_ERR_HIP;
}

granq_status_t granq_conv1x1_int8(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                  const int8_t *wq, const int32_t *corr, const float *out_scale,
                                  int bits, float *y, void *stream) {
    if (!desc || !codes || !wq || !corr || !out_scale || !y) return GRANQ_ERR_INVALID_ARG;
    if (desc->n <= 0 || desc->c <= 0 || desc->h <= 0 || desc->w <= 0 || o <= 0) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    const int64_t c = desc->c, hw = desc->h * desc->w, n = desc->n;
    // |sum| <= 127 * 255 * C must stay inside int32
    if (c >= ((int64_t)1 << 16) || o >= 65536 || n >= 65536 || hw >= ((int64_t)1 << 40)) return GRANQ_ERR_UNSUPPORTED;
    if (((uintptr_t)corr & 3u) || ((uintptr_t)out_scale & 3u) || ((uintptr_t)y & 3u)) return GRANQ_ERR_UNSUPPORTED;
    hipStream_t hs = (hipStream_t)stream;
    const bool mfma = bits <= 7 && c % 16 == 0 && o % 32 == 0 && hw % 4 == 0 &&
                      ((uintptr_t)codes & 3u) == 0 && ((uintptr_t)wq & 7u) == 0 && ((uintptr_t)y & 15u) == 0;
    if (mfma) {
        dim3 grid((uint32_t)((hw + 128 * (kBlock / kWave) - 1) / (128 * (kBlock / kWave))), (uint32_t)n), block(kBlock);
        int64_t ob = 0;
        while (ob < o) {                               // 64 output channels per launch, then 32
            if (o - ob >= 64) {
                hipLaunchKernelGGL(conv1x1_i8_mfma<2>, grid, block, 0, hs, codes, wq, corr, out_scale, y, c, hw, o, ob);
                ob += 64;
            } else {
                hipLaunchKernelGGL(conv1x1_i8_mfma<1>, grid, block, 0, hs, codes, wq, corr, out_scale, y, c, hw, o, ob);
                ob += 32;
            }
            if (hipGetLastError() != hipSuccess) return GRANQ_ERR_HIP;
        }
        return GRANQ_OK;
    }
    dim3 grid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)o, (uint32_t)n), block(kBlock);
    hipLaunchKernelGGL(conv1x1_i8_plain, grid, block, 0, hs, codes, wq, corr, out_scale, y, c, hw, o);
    return hipGetLastError() == hipSuccess ? GRANQ_OK : GRANQ_ERR_HIP;
}

}  // extern "C"
