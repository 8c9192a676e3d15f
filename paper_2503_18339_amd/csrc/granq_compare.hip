// Comparison points for the benchmark (see include/granq_compare.h): the
// channel-by-channel loop of the paper's Sec. 5.3.2 baseline, and the two
// accumulation forms of Eq. 3 and Eq. 6.  Deliberately plain kernels; the
// arithmetic is the same binary32 sequence as in the library.
#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

#include "granq_compare.h"
#include "granq_device.h"
#include "granq_launch.h"

namespace granq {

// One block per sample n: min/max of slab (n, ic); partial to ws[n], ws[N + n].
__global__ __launch_bounds__(kBlock) void cmp_range_one_channel(
    const float *__restrict__ x, int64_t c, int64_t hw, int64_t ic, int64_t n,
    float *__restrict__ ws)
{
    __shared__ float part[2][kBlock / kWave];
    const int64_t in = blockIdx.x;
    const float *slab = x + (in * c + ic) * hw;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int64_t k = threadIdx.x; k < hw; k += kBlock) {
        float v = slab[k];
        mn = __builtin_fminf(mn, v);
        mx = __builtin_fmaxf(mx, v);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { part[0][wave] = mn; part[1][wave] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) {
            mn = __builtin_fminf(mn, part[0][w]);
            mx = __builtin_fmaxf(mx, part[1][w]);
        }
        ws[in] = mn;
        ws[n + in] = mx;
    }
}

// One wavefront: fold the N partials of this one channel.
__global__ __launch_bounds__(kWave) void cmp_finish_one_channel(
    const float *__restrict__ ws, int64_t n, int64_t ic,
    float *__restrict__ ch_min, float *__restrict__ ch_max)
{
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int64_t i = threadIdx.x; i < n; i += kWave) {
        mn = __builtin_fminf(mn, ws[i]);
        mx = __builtin_fmaxf(mx, ws[n + i]);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if (threadIdx.x == 0) {
        ch_min[ic] = mn;
        ch_max[ic] = mx;
    }
}

__global__ void cmp_prescale_one_channel(const float *__restrict__ ch_min,
                                         const float *__restrict__ ch_max, int64_t ic, float qmax,
                                         float *__restrict__ scale, float *__restrict__ zero_point)
{
    const float mn = ch_min[ic];
    const float range = ch_max[ic] - mn;
    float s = range / qmax;
    if (!(s >= FLT_MIN)) s = 1.0f;
    scale[ic] = s;
    zero_point[ic] = __builtin_rintf((-mn) / s) + 0.0f;
}

// grid (chunks of hw, n): quantize-dequantize the slab (n, ic).
__global__ __launch_bounds__(kBlock) void cmp_fwd_one_channel(
    const float *x, float *x_hat, int64_t c, int64_t hw, int64_t ic,
    const float *__restrict__ scale, const float *__restrict__ zero_point, float qmax)
{
    const int64_t in = blockIdx.y;
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= hw) return;
    const float s = scale[ic], z = zero_point[ic];
    const int64_t at = (in * c + ic) * hw + k;
    const float q = clamp_code(raw_code(x[at], s, z), qmax);
    x_hat[at] = dequant(q, s, z);
}

// One thread per output pixel (n, k); channels in order, one rounding per operation.
__global__ __launch_bounds__(kBlock) void cmp_accumulate_inloop(
    const uint8_t *__restrict__ codes, int64_t c, int64_t hw, const float *__restrict__ scale,
    const float *__restrict__ zero_point, const float *__restrict__ weight, float *__restrict__ y)
{
    const int64_t in = blockIdx.y;
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= hw) return;
    const uint8_t *p = codes + in * c * hw + k;
    float acc = 0.0f;
    for (int64_t ic = 0; ic < c; ++ic) {
        const float d = (float)p[ic * hw] - zero_point[ic];
        const float ws = weight[ic] * scale[ic];       // the per-channel scaling, inside the loop
        const float term = ws * d;
        acc = acc + term;
    }
    y[in * hw + k] = acc;
}

__global__ __launch_bounds__(kBlock) void cmp_accumulate_prescaled(
    const float *__restrict__ x_hat, int64_t c, int64_t hw, const float *__restrict__ weight,
    float *__restrict__ y)
{
    const int64_t in = blockIdx.y;
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= hw) return;
    const float *p = x_hat + in * c * hw + k;
    float acc = 0.0f;
    for (int64_t ic = 0; ic < c; ++ic) {
        const float term = weight[ic] * p[ic * hw];
        acc = acc + term;
    }
    y[in * hw + k] = acc;
}

static granq_status_t cmp_check(const granq_desc_t *d) {
    if (!d) return GRANQ_ERR_INVALID_ARG;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0) return GRANQ_ERR_INVALID_ARG;
    if (d->dtype != GRANQ_F32) return GRANQ_ERR_UNSUPPORTED;
    // sample index rides on gridDim.y / gridDim.x
    if (d->n > 65535 || d->c >= ((int64_t)1 << 31) || d->h * d->w >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
    return GRANQ_OK;
}

static granq_status_t cmp_launched() {   // status of this call's own launches
    return launched();
}

}  // namespace granq

using namespace granq;

extern "C" {

granq_status_t granq_cmp_channel_loop_fwd(const float *x, const granq_desc_t *desc, int bits,
                                          float *ch_min, float *ch_max, float *scale,
                                          float *zero_point, float *x_hat, void *workspace,
                                          size_t workspace_bytes, void *stream) {
    granq_status_t st = cmp_check(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !ch_min || !ch_max || !scale || !zero_point || !x_hat) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < (size_t)(2 * desc->n) * sizeof(float) || ((uintptr_t)workspace & 15u))
        return GRANQ_ERR_WORKSPACE;
    hipStream_t hs = (hipStream_t)stream;
    const float qmax = (float)((1 << bits) - 1);
    const int64_t n = desc->n, c = desc->c, hw = desc->h * desc->w;
    float *ws = (float *)workspace;
    dim3 fgrid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)n);
    for (int64_t ic = 0; ic < c; ++ic) {               // the scalar loop over channels
        launch_kernel(cmp_range_one_channel, dim3((uint32_t)n), dim3(kBlock), 0, hs, x, c, hw, ic, n, ws);
        launch_kernel(cmp_finish_one_channel, dim3(1), dim3(kWave), 0, hs, ws, n, ic, ch_min, ch_max);
        launch_kernel(cmp_prescale_one_channel, dim3(1), dim3(1), 0, hs, ch_min, ch_max, ic, qmax, scale, zero_point);
        launch_kernel(cmp_fwd_one_channel, fgrid, dim3(kBlock), 0, hs, x, x_hat, c, hw, ic, scale, zero_point, qmax);
        st = cmp_launched();
        if (st != GRANQ_OK) return st;
    }
    return GRANQ_OK;
}

granq_status_t granq_cmp_accumulate_inloop(const uint8_t *codes, const granq_desc_t *desc,
                                           const float *scale, const float *zero_point,
                                           const float *weight, float *y, void *stream) {
    granq_status_t st = cmp_check(desc);
    if (st != GRANQ_OK) return st;
    if (!codes || !scale || !zero_point || !weight || !y) return GRANQ_ERR_INVALID_ARG;
    const int64_t hw = desc->h * desc->w;
    dim3 grid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)desc->n);
    launch_kernel(cmp_accumulate_inloop, grid, dim3(kBlock), 0, (hipStream_t)stream, codes, desc->c, hw, scale, zero_point, weight, y);
    return cmp_launched();
}

granq_status_t granq_cmp_accumulate_prescaled(const float *x_hat, const granq_desc_t *desc,
                                              const float *weight, float *y, void *stream) {
    granq_status_t st = cmp_check(desc);
    if (st != GRANQ_OK) return st;
    if (!x_hat || !weight || !y) return GRANQ_ERR_INVALID_ARG;
    const int64_t hw = desc->h * desc->w;
    dim3 grid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)desc->n);
    launch_kernel(cmp_accumulate_prescaled, grid, dim3(kBlock), 0, (hipStream_t)stream, x_hat, desc->c, hw, weight, y);
    return cmp_launched();
}

}  // extern "C"
