// Distortion metrics of the fake-quantized tensor (the paper's Table 2: cosine
// similarity and relative error between the activation X and its quantized
// version Q), fused with the quantizer: x is read once, Q = x_hat is recomputed
// in registers, four binary64 sums per channel come out.
//
// Pass 1: block (channel c, row group p); each wavefront takes whole (n,c) slabs,
// lanes stride over H*W (16-byte vectors, four in flight per lane, where the shape
// allows); per-lane binary64 accumulators, wavefront tree by
// shuffles, block tree through LDS, one partial per (p, c).  Pass 2: per channel
// and sum a wavefront adds the partials (lane-strided, then the shuffle tree); a last
// launch adds the channels the same way and forms the two ratios.  Every addition
// order is fixed, so the sums are reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_plan.h"
#include "granq_quotient.h"

namespace granq {

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// The four running sums of one lane, binary64.  FAST: the quotient of Eq. 1 through the
// channel's reciprocal r (granq_quotient.h: the same code u, five operations instead of a
// general division; it is arithmetic, not memory, that bounds this kernel).
struct Sums {
    double xq = 0.0, xx = 0.0, qq = 0.0, dd = 0.0;
    template <bool FAST>
    __device__ inline void add(float xf, float s, float z, float r, float qmax) {
        float u;
        if (FAST) u = __builtin_rintf(quotient_fast(quotient_clamp(xf), s, r) + z);
        else u = raw_code(xf, s, z);
        const float qf = dequant(clamp_code(u, qmax), s, z);
        const double xd = (double)xf, qd = (double)qf, d = xd - qd;
        xq += xd * qd;
        xx += xd * xd;
        qq += qd * qd;
        dd += d * d;
    }
};

// VECTOR: H*W is a whole number of 16-byte vectors and x is 16-byte aligned: a lane loads
// kMetricUnroll vectors of its slab at a time (non-temporally when STREAM: a tensor too
// large to stay cached) and adds their elements in index order.  Otherwise single elements.
constexpr int kMetricUnroll = 4;

template <typename T, bool VECTOR, bool STREAM>
__global__ __launch_bounds__(kBlock) void distortion_pass1(
    const void *__restrict__ x, const float *__restrict__ scale, const float *__restrict__ zero_point,
    float qmax, int64_t n, int64_t c, int64_t hw, RowPlan plan, double *__restrict__ ws)
{
    constexpr int VEC = T::VEC;
    using vec_t = typename T::vec_t;
    __shared__ double part[4][kBlock / kWave];
    const int64_t ic = blockIdx.x % c;
    const int64_t p = blockIdx.x / c;
    const int64_t r0 = p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < n) ? r0 + plan.rows_per_group : n;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const float s = scale[ic], z = zero_point[ic];
    const float r = 1.0f / s;
    Sums acc;
    auto sweep = [&](auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        for (int64_t in = r0 + wave; in < r1; in += kBlock / kWave) {
            const int64_t base = (in * c + ic) * hw;
            if (VECTOR) {
                const vec_t *row = (const vec_t *)x + base / VEC;
                const int64_t vecs = hw / VEC;
                for (int64_t k = lane; k < vecs; k += (int64_t)kWave * kMetricUnroll) {
                    vec_t v[kMetricUnroll];
#pragma unroll
                    for (int u = 0; u < kMetricUnroll; ++u)
                        if (k + u * kWave < vecs)
                            v[u] = STREAM ? __builtin_nontemporal_load(row + k + u * kWave) : row[k + u * kWave];
#pragma unroll
                    for (int u = 0; u < kMetricUnroll; ++u)
                        if (k + u * kWave < vecs) {
                            float f[VEC];
                            T::unpack(v[u], f);
#pragma unroll
                            for (int e = 0; e < VEC; ++e) acc.template add<FAST>(f[e], s, z, r, qmax);
                        }
                }
            } else {
                for (int64_t k = lane; k < hw; k += kWave) acc.template add<FAST>(T::load1(x, base + k), s, z, r, qmax);
            }
        }
    };
    if (quotient_fast_ok(s, z)) sweep(std::true_type{});     // block-uniform
    else sweep(std::false_type{});
    const double xq = wave_sum(acc.xq), xx = wave_sum(acc.xx), qq = wave_sum(acc.qq), dd = wave_sum(acc.dd);
    if (lane == 0) {
        part[0][wave] = xq;
        part[1][wave] = xx;
        part[2][wave] = qq;
        part[3][wave] = dd;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        double t = part[threadIdx.x][0];
        for (int w = 1; w < kBlock / kWave; ++w) t += part[threadIdx.x][w];
        ws[(p * c + ic) * 4 + threadIdx.x] = t;
    }
}

template <typename T>
static void launch_distortion_pass1(bool vector, bool stream, dim3 grid, hipStream_t hs, const void *x,
                                    const float *scale, const float *zero_point, float qmax, int64_t n,
                                    int64_t c, int64_t hw, RowPlan rp, double *ws) {
    dim3 block(kBlock);
    if (!vector)
        launch_kernel((distortion_pass1<T, false, false>), grid, block, 0, hs, x, scale, zero_point, qmax, n, c, hw, rp, ws);
    else if (stream)
        launch_kernel((distortion_pass1<T, true, true>), grid, block, 0, hs, x, scale, zero_point, qmax, n, c, hw, rp, ws);
    else
        launch_kernel((distortion_pass1<T, true, false>), grid, block, 0, hs, x, scale, zero_point, qmax, n, c, hw, rp, ws);
}

// Pass 2: block = channel, wavefront w = sum w of the four.  A lane adds the partials
// p = lane, lane + 64, ... in that order; the 64 lane sums then go through the shuffle tree.
__global__ __launch_bounds__(kBlock) void distortion_pass2(
    const double *__restrict__ ws, int64_t c, int32_t groups, double *__restrict__ ch_sums)
{
    static_assert(kBlock / kWave >= 4, "one wavefront per sum");
    const int64_t ic = blockIdx.x;
    const int which = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    if (which >= 4) return;
    double t = 0.0;
    for (int32_t p = lane; p < groups; p += kWave) t += ws[((int64_t)p * c + ic) * 4 + which];
    t = wave_sum(t);
    if (lane == 0) ch_sums[ic * 4 + which] = t;
}

// The whole tensor: wavefront w adds sum w of the channels (lane-strided, then the tree);
// thread 0 forms the two ratios.
__global__ __launch_bounds__(kBlock) void distortion_layer(const double *__restrict__ ch_sums, int64_t c,
                                                           double *__restrict__ layer)
{
    __shared__ double tot[4];
    const int which = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    double t = 0.0;
    if (which < 4)
        for (int64_t ic = lane; ic < c; ic += kWave) t += ch_sums[ic * 4 + which];
    t = wave_sum(t);
    if (lane == 0 && which < 4) {
        tot[which] = t;
        layer[which] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        layer[4] = tot[0] / (sqrt(tot[1]) * sqrt(tot[2]));      // X.Q / (|X| |Q|)
        layer[5] = sqrt(tot[3]) / sqrt(tot[1]);                 // |X - Q| / |X|
    }
}

// A tensor with a single channel (the layer-wise view {1,1,1,E}) is one slab, which one
// wavefront would have to walk alone.  All of it is channel 0, so it may be cut into any
// number of equal slabs: the largest power of two up to 4096 that divides the element count
// and leaves slabs that are still whole 16-byte vectors (or any slabs, for odd sizes).
static void fold_single_channel(int64_t &n, int64_t c, int64_t &hw, int vec) {
    if (c != 1) return;
    int64_t e = n * hw, r = 1;
    while (r < 4096 && e % (2 * r) == 0 && (e / (2 * r)) % vec == 0 && e / (2 * r) >= 4096) r *= 2;
    n = r;
    hw = e / r;
}

static granq_status_t metrics_check(const granq_desc_t *d) {
    if (!d) return GRANQ_ERR_INVALID_ARG;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0) return GRANQ_ERR_INVALID_ARG;
    if (d->dtype != GRANQ_F32 && d->dtype != GRANQ_BF16 && d->dtype != GRANQ_F16) return GRANQ_ERR_UNSUPPORTED;
    const int64_t lim = (int64_t)1 << 40;
    if (d->n > lim || d->c >= ((int64_t)1 << 24) || d->h > lim || d->w > lim || d->h * d->w > lim) return GRANQ_ERR_UNSUPPORTED;
    if ((__int128)d->n * d->c * (d->h * d->w) > ((__int128)1 << 46)) return GRANQ_ERR_UNSUPPORTED;
    return GRANQ_OK;
}

}  // namespace granq

using namespace granq;

extern "C" {

granq_status_t granq_distortion_workspace_bytes(const granq_desc_t *desc, size_t *bytes_out) {
    if (!bytes_out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = metrics_check(desc);
    if (st != GRANQ_OK) return st;
    int64_t n = desc->n, hw = desc->h * desc->w;
    fold_single_channel(n, desc->c, hw, desc->dtype == GRANQ_F32 ? 4 : 8);
    RowPlan rp = make_row_plan(n, desc->c, hw);
    *bytes_out = (size_t)rp.row_groups * (size_t)desc->c * 4 * sizeof(double);
    return GRANQ_OK;
}

granq_status_t granq_distortion(const void *x, const granq_desc_t *desc, const float *scale,
                                const float *zero_point, int bits, double *ch_sums, double *layer,
                                void *workspace, size_t workspace_bytes, void *stream) {
    granq_status_t st = metrics_check(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !scale || !zero_point || !ch_sums || !layer) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (((uintptr_t)x & (desc->dtype == GRANQ_F32 ? 3u : 1u)) || ((uintptr_t)scale & 3u) ||
        ((uintptr_t)zero_point & 3u) || ((uintptr_t)ch_sums & 7u) || ((uintptr_t)layer & 7u))
        return GRANQ_ERR_UNSUPPORTED;
    size_t need = 0;
    granq_distortion_workspace_bytes(desc, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u)) return GRANQ_ERR_WORKSPACE;
    hipStream_t hs = (hipStream_t)stream;
    int64_t n = desc->n, hw = desc->h * desc->w;
    fold_single_channel(n, desc->c, hw, desc->dtype == GRANQ_F32 ? 4 : 8);
    const float qmax = (float)((1 << bits) - 1);
    RowPlan rp = make_row_plan(n, desc->c, hw);
    double *ws = (double *)workspace;
    dim3 grid((uint32_t)(desc->c * rp.row_groups)), block(kBlock);
    const int esize = desc->dtype == GRANQ_F32 ? 4 : 2;
    const bool vector = hw % (16 / esize) == 0 && ((uintptr_t)x & 15u) == 0;
    const bool streamed = n * desc->c * hw * esize >= ((int64_t)256 << 20);   // beyond the memory-side cache
    if (desc->dtype == GRANQ_F32)
        launch_distortion_pass1<F32>(vector, streamed, grid, hs, x, scale, zero_point, qmax, n, desc->c, hw, rp, ws);
    else if (desc->dtype == GRANQ_BF16)
        launch_distortion_pass1<BF16>(vector, streamed, grid, hs, x, scale, zero_point, qmax, n, desc->c, hw, rp, ws);
    else
        launch_distortion_pass1<F16>(vector, streamed, grid, hs, x, scale, zero_point, qmax, n, desc->c, hw, rp, ws);
    if (launched() != GRANQ_OK) return GRANQ_ERR_HIP;
    launch_kernel(distortion_pass2, dim3((uint32_t)desc->c), block, 0, hs, ws, desc->c, rp.row_groups, ch_sums);
    if (launched() != GRANQ_OK) return GRANQ_ERR_HIP;
    launch_kernel(distortion_layer, dim3(1), block, 0, hs, ch_sums, desc->c, layer);
    return launched();
}

}  // extern "C"
